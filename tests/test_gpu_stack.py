"""Temporal stacking on the GPU (Section 5 of the paper: several meta-kernels merged into one launch).

The stacked launch must give, for every part, exactly the bits the part gives when launched alone
(same bytecode body, same interpreter arithmetic), and those match the oracle.
"""
from __future__ import annotations

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


def _bits(t):
    return t.contiguous().view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


_stack_ctx = None


def stack_ctx():
    """Parts that share a launch must fit one interpreter variant: encode all of them under common limits."""
    global _stack_ctx
    if _stack_ctx is None:
        _stack_ctx = B.Context(torch.cuda.current_device())
        _stack_ctx.set_limits(16, 6)
    return _stack_ctx


def run_stacked(parts, spatial=False):
    """parts: list of (desc, inputs dict, optional output views dict).  Returns per-part output dicts."""
    ctx = stack_ctx()
    codes, tensors, outs_all = [], [], []
    for desc, ins, views in parts:
        prog = H.program(desc)
        in_list = [ins[n] for n, _ in desc.inputs]
        if views is None:
            code = B.encode_for(ctx, prog, in_list)
            outs = [torch.zeros(s, dtype=H._TORCH_DT[dt], device=DEV) for (_, dt), s in zip(desc.outputs, code.out_shapes)]
        else:
            outs = [views[n] for n, _ in desc.outputs]
            code = B.encode_for(ctx, prog, in_list, outs)
        codes.append(code)
        tensors += in_list + outs
        outs_all.append({n: t for (n, _), t in zip(desc.outputs, outs)})
    stacked = B.dvm_stack(codes, spatial=spatial)
    stacked.validate()
    inf = stacked.info()
    assert inf.n_segments == len(parts)
    B.run_on(ctx, stacked, tensors)
    torch.cuda.synchronize()
    return outs_all, stacked


def check_parts(parts, what, spatial=False):
    stacked_outs, code = run_stacked(parts, spatial)
    for (desc, ins, views), got in zip(parts, stacked_outs):
        got = {k: v.clone() for k, v in got.items()}
        alone, _ = H.run_vm(desc, ins, views, ctx=stack_ctx())
        rounded, exact = H.run_oracle(desc, ins)
        for n, dt in desc.outputs:
            assert torch.equal(_bits(got[n]), _bits(alone[n])), f"{what}: {desc.name}:{n} differs from the single launch"
            H.compare(got[n], rounded[n], exact[n], dt, H.has_reduction(desc), f"{what}: {desc.name}:{n}")
    return code


@pytest.mark.parametrize("T", [1, 37, 700])
def test_c5_layer_in_one_launch(T):
    say(f"c5 layer stacked, T={T}")
    d = gen.c5_inputs(T, 900 + T, DEV)
    rope_out = torch.zeros((T, 32, 128), dtype=torch.bfloat16, device=DEV)
    parts = [
        (W.get_program("c5_rmsnorm"), d["c5_rmsnorm"], None),
        (W.get_program("c5_rope"), d["c5_rope"], {"y1": rope_out[..., :64], "y2": rope_out[..., 64:]}),
        (W.get_program("c5_softmax"), d["c5_softmax"], None),
        (W.get_program("c5_residual"), d["c5_residual_a"], None),
        (W.get_program("c5_silu_gate"), d["c5_silu_gate"], None),
        (W.get_program("c5_residual"), d["c5_residual_b"], None),
    ]
    code = check_parts(parts, f"c5 T={T}")
    assert "vstack.t" in code.disasm()
    # the same layer with its six programs side by side on shares of the workgroups (spatial stacking)
    for _, _, views in parts:
        if views:
            for v in views.values():
                v.zero_()
    code = check_parts(parts, f"c5 spatial T={T}", spatial=True)
    assert "vstack.s" in code.disasm()


def test_stack_of_different_shapes_and_variants():
    say("stack: rmsnorm instances of different sizes + fp32 program with short rows")
    parts = []
    for i, (b, s) in enumerate([(1, 3), (2, 515), (1, 64), (3, 1000)]):
        parts.append((W.get_program("c2_rmsnorm"), gen.c2_inputs(b, s, 950 + i, DEV), None))
    parts.append((W.get_program("c1_gelu_erf"), gen.c1_inputs(960, DEV), None))
    z = gen.randn((4, 33, 100), 961, DEV, "f32", std=3.0)
    parts.append((W.get_program("softmax_f32"), {"z": z}, None))
    check_parts(parts, "mixed stack")
    check_parts(parts, "mixed stack, spatial", spatial=True)


def test_stack_limits():
    ctx = stack_ctx()
    prog = H.program(W.get_program("c2_rmsnorm"))
    d = gen.c2_inputs(1, 8, 970, DEV)
    code = B.encode_for(ctx, prog, [d["x"], d["w"]])
    with pytest.raises(B.DvmError):
        B.dvm_stack([code] * 11)        # 33 tensors: beyond the launch's tensor table
