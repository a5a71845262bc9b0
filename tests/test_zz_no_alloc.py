"""dvm_run_static: the entry point for callers that cannot allocate device memory.  A dependent stack with a
grid-wide synchronisation point runs through it (the library's own device array is the workspace) and must give
exactly the bits dvm_run gives with a workspace of the caller's: two calls in a row, the second on a smaller input."""
from __future__ import annotations

import ctypes as C

import pytest
import torch

from paper_2603_24239_amd import binding as B
from workloads import gen
from workloads import programs as W
from workloads.programs import _p, single_op_program

from . import harness as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _bits(t):
    return t.contiguous().view(torch.int16)


def _case(ctx, T, seed):
    """rmsnorm -> add over another view of its output -> softmax: two grid-wide waits."""
    d = gen.c5_inputs(T, seed, DEV)["c5_rmsnorm"]
    norm = W.get_program("c5_rmsnorm")
    add = single_op_program("add", 2, "bf16")
    soft = _p("soft_bf16", [("z", "bf16")], [("y", "softmax", ["z"], {})], [("y", "bf16")])
    other = gen.randn((T * 4, 1024), seed + 7, DEV, "bf16")
    ins = [d[n] for n, _ in norm.inputs]

    def buffers():
        return [torch.zeros((T, 4096), dtype=torch.bfloat16, device=DEV), torch.zeros((T * 4, 1024), dtype=torch.bfloat16, device=DEV),
                torch.zeros((T, 4096), dtype=torch.bfloat16, device=DEV)]

    y, s, p = buffers()
    codes = [B.encode_for(ctx, H.program(norm), ins, [y]),
             B.encode_for(ctx, H.program(add), [y.view(T * 4, 1024), other], [s]),
             B.encode_for(ctx, H.program(soft), [s.view(T, 4096)], [p])]
    st = B.dvm_stack_dependent(codes, [-1, -1, -1, 2, -1, -1, 5, -1])
    assert st.needs_workspace() and st.info().n_tensors == 9

    def tensors(y, s, p):
        return [t.data_ptr() for t in ins + [y, y, other, s, s, p]]

    return st, buffers, tensors


def test_static_workspace_entry_point_matches_dvm_run_on_two_calls_in_a_row():
    print("[case] dvm_run_static vs dvm_run, T=3000 then T=41", flush=True)
    ctx = B.Context(torch.cuda.current_device())
    ctx.set_limits(16, 6)
    stream = torch.cuda.current_stream().cuda_stream
    ws = torch.empty(B.WORKSPACE_BYTES // 4, dtype=torch.int32, device=DEV)
    for T, seed in ((3000, 5100), (41, 5200)):
        st, buffers, tensors = _case(ctx, T, seed)
        want = buffers()
        B.dvm_run(ctx, st, tensors(*want) + [ws.data_ptr()], stream)
        assert not B.workspace_gave_up(ws.data_ptr(), stream)
        got = buffers()
        B.dvm_run_static(ctx, st, tensors(*got), stream)        # one entry fewer: no workspace
        torch.cuda.synchronize()
        for g, w_, name in zip(got, want, ("rmsnorm", "add", "softmax")):
            assert torch.equal(_bits(g), _bits(w_)), f"T={T}: {name} differs between dvm_run_static and dvm_run"
        assert float(got[2].float().sum(dim=-1).sub(1).abs().max()) < 0.05          # (rows of a softmax)
    # argument errors: the workspace entry must be left out; bytecode without workspace runs as with dvm_run
    st, buffers, tensors = _case(ctx, 8, 5300)
    b = buffers()
    with pytest.raises(B.DvmError):
        B.dvm_run_static(ctx, st, tensors(*b) + [ws.data_ptr()], stream)
    norm = W.get_program("c5_rmsnorm")
    d = gen.c5_inputs(8, 5400, DEV)["c5_rmsnorm"]
    ins = [d[n] for n, _ in norm.inputs]
    code = B.encode_for(ctx, H.program(norm), ins)
    y1 = torch.zeros((8, 4096), dtype=torch.bfloat16, device=DEV)
    y2 = torch.zeros_like(y1)
    B.dvm_run(ctx, code, [t.data_ptr() for t in ins + [y1]], stream)
    B.dvm_run_static(ctx, code, [t.data_ptr() for t in ins + [y2]], stream)
    torch.cuda.synchronize()
    assert torch.equal(_bits(y1), _bits(y2))
