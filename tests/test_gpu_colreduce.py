"""Parity of reductions along the penultimate axis (Table 1's Sum / Max / Min over [M, size, N] with N > 1)
against the oracle: element by element, fp32 rtol 1e-4 (the tolerance of programs with a reduction)."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2603_24239_amd import binding as B
from workloads import gen
from workloads import programs as W

from . import harness as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[case] {msg}", flush=True)


def randn(shape, seed, dtype=torch.float32, scale=1.0):
    g = torch.Generator(device="cpu").manual_seed(gen.BASE_SEED + seed)
    return (torch.randn(shape, generator=g, dtype=torch.float32) * scale).to(dtype).to(DEV)


def check(desc, ins, what):
    outs, code = H.run_vm(desc, ins)
    rounded, exact = H.run_oracle(desc, ins)
    for n, dt in desc.outputs:
        H.compare(outs[n], rounded[n], exact[n], dt, True, f"{what}:{n}")
    return outs, code


# several units per workgroup, ragged row tails, one and several column tiles, rank 2 to 4, a short reduced axis
SHAPES = [(3, 37, 300), (5, 7, 33), (1, 1000, 4096), (2, 64, 8200), (513, 1024), (2, 3, 17, 129), (600, 2, 8),
          (1, 4097, 5), (700, 3, 64)]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_colsum_matches_oracle(shape):
    say(f"colsum {shape}")
    x = randn(shape, 7000 + len(shape) + shape[-1])
    outs, code = check(W.get_program("colsum"), {"x": x}, f"colsum{shape}")
    assert tuple(outs["s"].shape) == tuple(shape[:-2]) + (1, shape[-1])


@pytest.mark.parametrize("shape", [(3, 50, 256), (1, 333, 1030), (64, 9, 40)], ids=lambda s: "x".join(map(str, s)))
def test_col_stats_epilogue_matches_oracle(shape):
    say(f"col_stats {shape}")
    x = randn(shape, 7100 + shape[-1])
    b = randn((shape[-1],), 7101)
    check(W.get_program("col_stats"), {"x": x, "b": b}, f"col_stats{shape}")


def test_full_size_output_beside_the_reduction():
    say("colsum_exp (1500, 700)")
    x = randn((1500, 700), 7200, scale=0.5)
    check(W.get_program("colsum_exp"), {"x": x}, "colsum_exp")


def test_bias_gradient_bf16_at_layer_size():
    # [tokens, hidden] bf16 -> [1, hidden] fp32, the oracle evaluates it whole
    say("bias_grad_bf16 (8192, 4096)")
    dy = randn((8192, 4096), 7300, dtype=torch.bfloat16)
    check(W.get_program("bias_grad_bf16"), {"dy": dy}, "bias_grad")


def test_strided_rows_and_extent_one_axis():
    say("colsum on every second row of [4, 40, 96]; colsum over an axis of extent 1")
    base = randn((4, 40, 96), 7400)
    check(W.get_program("colsum"), {"x": base[:, ::2, :]}, "colsum strided")
    one = randn((9, 1, 130), 7401)
    outs, _ = check(W.get_program("colsum"), {"x": one}, "colsum extent 1")
    assert torch.equal(outs["s"], one)


def test_stacked_with_a_row_program():
    # temporal stacking: the column reduction shares a launch (and a larger workgroup) with an RMSNorm
    say("stack colsum + c2_rmsnorm")
    # (a context limited to 16 elements per lane, and enough units that one wave takes each: the stacked
    # launch runs the variant that holds every part, at the largest workgroup of the parts)
    ctx = B.Context(torch.cuda.current_device())
    ctx.set_limits(16, 6)
    x = randn((8000, 5, 200), 7500)
    d = gen.c2_inputs(1, 64, gen.BASE_SEED + 7501, DEV)
    pa, pb = H.program(W.get_program("colsum")), H.program(W.get_program("c2_rmsnorm"))
    ca = B.encode_for(ctx, pa, [x])
    cb = B.encode_for(ctx, pb, [d["x"], d["w"]])
    s = torch.empty(ca.out_shapes[0], dtype=torch.float32, device=DEV)
    y = torch.empty(cb.out_shapes[0], dtype=torch.bfloat16, device=DEV)
    for spatial in (False, True):       # one after the other in every workgroup, then side by side on shares of them
        st = B.dvm_stack([ca, cb], spatial=spatial)
        s.fill_(float("nan")); y.fill_(float("nan"))
        B.run_on(ctx, st, [x, s, d["x"], d["w"], y])
        torch.cuda.synchronize()
        for desc, ins, out, name in ((W.get_program("colsum"), {"x": x}, s, "s"), (W.get_program("c2_rmsnorm"), d, y, "y")):
            rounded, exact = H.run_oracle(desc, ins)
            H.compare(out, rounded[name], exact[name], desc.outputs[0][1], True, f"stacked {desc.name} spatial={spatial}")


@pytest.mark.parametrize("waves", [1, 3, 16])
def test_any_number_of_waves_per_unit(waves):
    # the planner picks the waves that share a unit; the debug override walks the other settings,
    # among them one wave (no combination step) and a count that does not divide the reduced extent
    say(f"col_stats with {waves} wave(s) per unit")
    ctx = B.Context(torch.cuda.current_device())
    ctx.set_plan_override(rows_per_tile=waves)
    desc = W.get_program("col_stats")
    ins = {"x": randn((5, 37, 300), 7600 + waves), "b": randn((300,), 7601)}
    outs, code = H.run_vm(desc, ins, ctx=ctx)
    assert code.info().block == 64 * waves
    rounded, exact = H.run_oracle(desc, ins)
    for n, dt in desc.outputs:
        H.compare(outs[n], rounded[n], exact[n], dt, True, f"col_stats waves={waves}:{n}")


def _prog(name, inputs, ops, outputs):
    from workloads.programs import _p
    return _p(name, inputs, ops, outputs)


def test_broadcast_operands_before_and_after_the_reduction():
    # a weight per reduced row ([size, 1]: a row value in the per-row part), a bias per column added before the
    # reduction, and a scale per outer index ([M, 1, 1]: a row value in the epilogue)
    say("weighted column sum with bias and per-index scale, fp32 [5, 41, 700]")
    desc = _prog("weighted_colsum", [("x", "f32"), ("w", "f32"), ("b", "f32"), ("g", "f32")],
                 [("t", "add", ["x", "b"], {}), ("u", "mul", ["t", "w"], {}), ("s", "csum", ["u"], {}),
                  ("y", "mul", ["s", "g"], {})], [("y", "f32")])
    ins = {"x": randn((5, 41, 700), 7700), "w": randn((41, 1), 7701), "b": randn((700,), 7702), "g": randn((5, 1, 1), 7703)}
    check(desc, ins, "weighted_colsum")


@pytest.mark.parametrize("shape", [(3, 29, 520), (1, 257, 72), (40, 6, 4096)], ids=lambda s: "x".join(map(str, s)))
def test_bf16_storage(shape):
    # bf16 in and out (chunks of eight elements): max and min are exact, the sum is rounded once at the output
    say(f"bf16 column max / min / sum {shape}")
    desc = _prog("col_bf16", [("x", "bf16")],
                 [("hi", "cmax", ["x"], {}), ("lo", "cmin", ["x"], {}), ("s", "csum", ["x"], {})],
                 [("hi", "bf16"), ("lo", "bf16"), ("s", "bf16")])
    x = randn(shape, 7800 + shape[-1], dtype=torch.bfloat16)
    outs, _ = check(desc, {"x": x}, f"col_bf16{shape}")
    assert torch.equal(outs["hi"], x.max(dim=-2, keepdim=True).values)
    assert torch.equal(outs["lo"], x.min(dim=-2, keepdim=True).values)


def test_empty_outer_extent_launches_nothing():
    say("colsum [0, 5, 7]")
    x = torch.empty((0, 5, 7), dtype=torch.float32, device=DEV)
    outs, code = H.run_vm(W.get_program("colsum"), {"x": x})
    assert tuple(outs["s"].shape) == (0, 1, 7) and code.info().n_tiles == 0


def test_stacked_under_a_larger_workgroup():
    # four waves share a unit; the stacked launch runs sixteen waves per workgroup (a softmax over rows of 8192
    # elements at eight elements per lane): the twelve waves outside the reduction's workgroup hold no rows but
    # take part in its combination step's synchronisation
    say("stack colsum (4 waves per unit) + softmax_f32 rows of 8192 (1024 threads)")
    ctx = B.Context(torch.cuda.current_device())
    ctx.set_plan_override(rows_per_tile=4)
    ctx.set_limits(8, 6)
    x = randn((12, 70, 520), 7900)
    z = randn((24, 8192), 7901)
    pa, pb = H.program(W.get_program("colsum")), H.program(W.get_program("softmax_f32"))
    ca = B.encode_for(ctx, pa, [x])
    cb = B.encode_for(ctx, pb, [z])
    assert ca.info().block == 256 and cb.info().block == 1024
    s = torch.empty(ca.out_shapes[0], dtype=torch.float32, device=DEV)
    p = torch.empty(cb.out_shapes[0], dtype=torch.float32, device=DEV)
    for order in ((ca, cb), (cb, ca)):
        st = B.dvm_stack(list(order))
        assert st.info().block == 1024
        s.fill_(float("nan")); p.fill_(float("nan"))
        B.run_on(ctx, st, [x, s, z, p] if order[0] is ca else [z, p, x, s])
        torch.cuda.synchronize()
        for desc, ins, out, name in ((W.get_program("colsum"), {"x": x}, s, "s"), (W.get_program("softmax_f32"), {"z": z}, p, "p")):
            rounded, exact = H.run_oracle(desc, ins)
            H.compare(out, rounded[name], exact[name], "f32", True, f"stacked {desc.name}")


@pytest.mark.parametrize("op", ["cmax", "cmin", "csum"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_single_reduction_of_an_input_streams(op, dtype):
    # nothing but the reduction of an input: the streaming record (several rows in flight per wave); max and min
    # are exact in both storage types
    from workloads.programs import single_op_program
    shape = (3, 77, 1100)
    say(f"{op} {dtype} {shape}")
    desc = single_op_program(op, 1, dtype)
    x = randn(shape, 8100 + len(op), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32)
    outs, code = check(desc, {"a0": x}, f"{op} {dtype}")
    assert "stream." in code.disasm()
    if op == "cmax":
        assert torch.equal(outs["y"], x.max(dim=-2, keepdim=True).values)
    if op == "cmin":
        assert torch.equal(outs["y"], x.min(dim=-2, keepdim=True).values)
