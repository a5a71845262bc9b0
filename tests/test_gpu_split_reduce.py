"""Reductions along the penultimate axis split over a workspace (Table 1's Sum / Max / Min over [M, size, N] with few
(M, column tile) units and a long `size`): S row ranges leave partial results in the workspace, a second meta-kernel,
launched behind the first, combines them.  Parity with the oracle, the same bits on every run, dvm_run_static."""
from __future__ import annotations

import pytest
import torch

from paper_2603_24239_amd import binding as B
from workloads import gen
from workloads.programs import _p

from . import harness as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[case] {msg}", flush=True)


def _ctx():
    c = B.Context(torch.cuda.current_device())
    c.set_workspace_limit(4 << 20)
    return c


def _run(ctx, desc, ins, static=False):
    prog = H.program(desc)
    in_list = [ins[n] for n, _ in desc.inputs]
    code = B.encode_for(ctx, prog, in_list)
    outs = [torch.full(s, float("nan"), dtype=H._TORCH_DT[dt], device=DEV) for (_, dt), s in zip(desc.outputs, code.out_shapes)]
    ptrs = [t.data_ptr() for t in in_list + outs]
    stream = torch.cuda.current_stream().cuda_stream
    if code.needs_workspace() and not static:
        need = code.tensor(code.info().n_tensors - 1)[0]
        ws = torch.full((need // 4,), -1, dtype=torch.int32, device=DEV)
        B.dvm_run(ctx, code, ptrs + [ws.data_ptr()], stream)      # (no device-side wait in such a program: no status to read)
    elif code.needs_workspace():
        B.dvm_run_static(ctx, code, ptrs, stream)
    else:
        B.dvm_run(ctx, code, ptrs, stream)
    torch.cuda.synchronize()
    return {n: t for (n, _), t in zip(desc.outputs, outs)}, code


CASES = [
    ("bias gradient", _p("biasgrad", [("g", "f32")], [("s", "csum", ["g"], {})], [("s", "f32")]), [(8192, 4096)], ["f32"]),
    ("bias gradient bf16", _p("biasgrad16", [("g", "bf16")], [("s", "csum", ["g"], {})], [("s", "f32")]), [(4096, 1000)], ["bf16"]),
    ("column max, ragged columns", _p("cmax", [("x", "f32")], [("m", "cmax", ["x"], {})], [("m", "f32")]), [(3, 2048, 333)], ["f32"]),
    ("log-sum-exp over rows plus a bias", _p("lse", [("x", "bf16"), ("b", "f32")],
                                             [("e", "exp", ["x"], {}), ("s", "csum", ["e"], {}), ("l", "log", ["s"], {}), ("y", "add", ["l", "b"], {})],
                                             [("y", "f32")]), [(2, 4096, 1000), (2, 1, 1000)], ["bf16", "f32"]),
    ("column min of a product", _p("cminprod", [("a", "f32"), ("w", "f32")], [("p", "mul", ["a", "w"], {}), ("m", "cmin", ["p"], {})],
                                   [("m", "bf16")]), [(1, 6000, 520), (520,)], ["f32", "f32"]),
]


@pytest.mark.parametrize("what,desc,shapes,dts", CASES, ids=[c[0] for c in CASES])
def test_split_reduction_matches_the_oracle_and_itself(what, desc, shapes, dts):
    say(f"split reduction: {what} {shapes}")
    ctx = _ctx()
    ins = {n: gen.randn(sh, 8100 + i, DEV, dt) for i, ((n, _), sh, dt) in enumerate(zip(desc.inputs, shapes, dts))}
    outs, code = _run(ctx, desc, ins)
    txt = code.disasm()
    assert code.needs_workspace() and "vstack.t" in txt and "a kernel launch of its own" in txt, txt
    rounded, exact = H.run_oracle(desc, ins)
    for n, dt in desc.outputs:
        H.compare(outs[n], rounded[n], exact[n], dt, True, f"{what}: {n}")
    # the same bits on a second run and through the entry point that brings its own workspace
    again, _ = _run(ctx, desc, ins)
    static, _ = _run(ctx, desc, ins, static=True)
    for n, _dt in desc.outputs:
        assert torch.equal(outs[n].view(torch.int16 if outs[n].dtype == torch.bfloat16 else torch.int32),
                           again[n].view(torch.int16 if outs[n].dtype == torch.bfloat16 else torch.int32)), f"{what}: {n} differs between runs"
        assert torch.equal(outs[n].view(torch.int16 if outs[n].dtype == torch.bfloat16 else torch.int32),
                           static[n].view(torch.int16 if outs[n].dtype == torch.bfloat16 else torch.int32)), f"{what}: {n} differs with the static workspace"


def test_programs_that_do_not_split_need_no_workspace():
    ctx = _ctx()
    many_units = _p("cs", [("x", "f32")], [("s", "csum", ["x"], {})], [("s", "f32")])
    x = gen.randn((256, 64, 1024), 8200, DEV)                   # plenty of units already
    outs, code = _run(ctx, many_units, {"x": x})
    assert not code.needs_workspace()
    rounded, exact = H.run_oracle(many_units, {"x": x})
    H.compare(outs["s"], rounded["s"], exact["s"], "f32", True, "unsplit column sum")
    # a full-size output beside the reduction: not split (its rows would have to be written by the first part)
    both = _p("e_and_s", [("x", "f32")], [("e", "exp", ["x"], {}), ("s", "csum", ["e"], {})], [("e", "f32"), ("s", "f32")])
    x = gen.randn((1, 4096, 512), 8201, DEV)
    outs, code = _run(ctx, both, {"x": x})
    assert not code.needs_workspace()
    # without a workspace limit nothing is ever split
    plain = B.Context(torch.cuda.current_device())
    g = gen.randn((8192, 512), 8202, DEV)
    code = B.encode_for(plain, H.program(many_units), [g])
    assert not code.needs_workspace()
