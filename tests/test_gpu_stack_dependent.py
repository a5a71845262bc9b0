"""Temporal stacking of parts that depend on each other, on the GPU (Section 5.1: stacking does not require
independent operators; Section 5.2: the pieces of an unmergeable sequence run as one stacked kernel).

One launch runs a producer and its consumers.  Every part's outputs must have exactly the bits the same parts give
when launched one after the other, and every part must match the oracle applied to the inputs that part really saw
(for a consumer: the producer's output as it stands in memory)."""
from __future__ import annotations

import pytest
import torch

from paper_2603_24239_amd import binding as B
from workloads import gen
from workloads import programs as W
from workloads.programs import _p, single_op_program

from . import harness as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[case] {msg}", flush=True)


def _bits(t):
    return t.contiguous().view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


_ctx = None


def dep_ctx():
    global _ctx
    if _ctx is None:
        _ctx = B.Context(torch.cuda.current_device())
        _ctx.set_limits(16, 6)
    return _ctx


def run_chain(parts, one_launch=True, ctx=None, order_by="kernel"):
    """parts: list of (desc, {input name: tensor}, {output name: tensor} or None for fresh zeroed outputs).  An input
    at the address of an earlier part's output is that buffer.  Returns (outputs per part, the stacked bytecode)."""
    ctx = ctx or dep_ctx()
    codes, tensors, outs_all = [], [], []
    for desc, ins, given in parts:
        in_list = [ins[n] for n, _ in desc.inputs]
        prog = H.program(desc)
        if given is None:
            code = B.encode_for(ctx, prog, in_list)
            outs = [torch.zeros(s, dtype=H._TORCH_DT[dt], device=DEV) for (_, dt), s in zip(desc.outputs, code.out_shapes)]
        else:
            outs = [given[n] for n, _ in desc.outputs]
            code = B.encode_for(ctx, prog, in_list, outs)
        codes.append(code)
        tensors.append(in_list + outs)
        outs_all.append({n: t for (n, _), t in zip(desc.outputs, outs)})
    if not one_launch:
        for code, ts in zip(codes, tensors):
            B.run_on(ctx, code, ts)
        torch.cuda.synchronize()
        return outs_all, None
    flat = [t for ts in tensors for t in ts]
    # entries with the same address are the same buffer (the parts here never share part of a buffer only)
    same_as = [next((j for j in range(i) if flat[j].data_ptr() == t.data_ptr()), -1) for i, t in enumerate(flat)]
    st = B.dvm_stack_dependent(codes, same_as, order_by)
    st.validate()
    ptrs = [t.data_ptr() for t in flat]
    if st.needs_workspace():
        ws = torch.full((B.WORKSPACE_BYTES // 4,), -1, dtype=torch.int32, device=DEV)      # (dvm_run clears it)
        ptrs.append(ws.data_ptr())
        B.dvm_run(ctx, st, ptrs, torch.cuda.current_stream().cuda_stream)
        assert not B.workspace_gave_up(ws.data_ptr(), torch.cuda.current_stream().cuda_stream)
    else:
        B.dvm_run(ctx, st, ptrs, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return outs_all, st


def check_chain(build, what, expect):
    """build(): a fresh list of parts (fresh output buffers).  Runs it as one launch and as one launch per part."""
    parts = build()
    got, st = run_chain(parts)
    txt = st.disasm()
    for needle, count in expect.items():
        assert txt.count(needle) == count, (what, needle, txt)
    parts2 = build()
    alone, _ = run_chain(parts2, one_launch=False)
    # the same program with launch boundaries instead of waits on the device
    parts3 = build()
    by_launch, st3 = run_chain(parts3, order_by="launch")
    assert not st3.needs_workspace() and st3.info().n_launches == 1 + txt.count(GRID)
    for (desc, _, _), g, b3 in zip(parts, got, by_launch):
        for n, _dt in desc.outputs:
            assert torch.equal(_bits(g[n]), _bits(b3[n])), f"{what}: {desc.name}:{n} differs between the two ways of ordering the parts"
    for (desc, ins, _), g, a in zip(parts, got, alone):
        rounded, exact = H.run_oracle(desc, ins)       # (ins hold what the stacked launch left in memory)
        for n, dt in desc.outputs:
            assert torch.equal(_bits(g[n]), _bits(a[n])), f"{what}: {desc.name}:{n} differs from launching the parts in order"
            H.compare(g[n], rounded[n], exact[n], dt, H.has_reduction(desc), f"{what}: {desc.name}:{n}")
    return st


WG = "waits for this workgroup's own stores"
GRID = "waits until every workgroup has finished"
SOFT_BF16 = _p("soft_bf16", [("z", "bf16")], [("y", "softmax", ["z"], {})], [("y", "bf16")])


@pytest.mark.parametrize("T", [1, 37, 3000])
def test_rmsnorm_feeds_softmax_same_rows(T):
    say(f"dependent stack, same rows per workgroup: rmsnorm -> softmax, T={T}")

    def build():
        d = gen.c5_inputs(T, 4100 + T, DEV)["c5_rmsnorm"]
        y = torch.zeros((T, 4096), dtype=torch.bfloat16, device=DEV)
        return [(W.get_program("c5_rmsnorm"), d, {"y": y}), (SOFT_BF16, {"z": y}, None)]

    check_chain(build, f"rmsnorm->softmax T={T}", {WG: 1, GRID: 0})


@pytest.mark.parametrize("T", [1, 37, 3000])
def test_dependent_c5_layer_in_one_launch(T):
    """A transformer layer's non-GEMM programs with their real dependences: the first residual's output feeds the
    RMSNorm and the second residual; RoPE, softmax and the gated activation ride along."""
    say(f"dependent c5 layer, T={T}")

    def build():
        d = gen.c5_inputs(T, 4200 + T, DEV)
        res, norm = W.get_program("c5_residual"), W.get_program("c5_rmsnorm")
        names_r = [n for n, _ in res.inputs]
        h = torch.zeros((T, 4096), dtype=torch.bfloat16, device=DEV)
        rope_out = torch.zeros((T, 32, 128), dtype=torch.bfloat16, device=DEV)
        ra = d["c5_residual_a"]
        rb = dict(d["c5_residual_b"])
        rb[names_r[0]] = h
        nin = dict(d["c5_rmsnorm"])
        nin[norm.inputs[0][0]] = h
        return [
            (res, ra, {res.outputs[0][0]: h}),
            (norm, nin, None),
            (W.get_program("c5_rope"), d["c5_rope"], {"y1": rope_out[..., :64], "y2": rope_out[..., 64:]}),
            (W.get_program("c5_softmax"), d["c5_softmax"], None),
            (W.get_program("c5_silu_gate"), d["c5_silu_gate"], None),
            (res, rb, None),
        ]

    st = check_chain(build, f"dependent c5 layer T={T}", {})
    txt = st.disasm()
    assert txt.count(WG) + txt.count(GRID) == 2 and st.info().n_segments == 6


@pytest.mark.parametrize("T", [5, 2000])
def test_consumer_with_other_tiles_uses_the_grid_wide_wait(T):
    say(f"dependent stack, grid-wide wait: rmsnorm -> add over another view -> column sum, T={T}")

    def build():
        d = gen.c5_inputs(T, 4300 + T, DEV)["c5_rmsnorm"]
        y = torch.zeros((T, 4096), dtype=torch.bfloat16, device=DEV)
        other = gen.randn((T * 4, 1024), 4301 + T, DEV, "bf16")
        s = torch.zeros((T * 4, 1024), dtype=torch.bfloat16, device=DEV)
        add = single_op_program("add", 2, "bf16")
        return [(W.get_program("c5_rmsnorm"), d, {"y": y}),
                (add, {"a0": y.view(T * 4, 1024), "a1": other}, {"y": s}),
                (SOFT_BF16, {"z": s.view(T, 4096)}, None)]

    check_chain(build, f"grid-wide T={T}", {WG: 0, GRID: 2})


def test_bounded_wait_gives_up_and_the_next_launch_recovers():
    """With the poll limit at its minimum the first workgroup to reach the synchronisation point abandons it; the
    status word says so, every workgroup leaves the kernel, and the next launch (default limit) is unaffected."""
    say("grid-wide wait with a poll limit of 1, then the default")
    T = 8192
    ctx = B.Context(torch.cuda.current_device())
    ctx.set_limits(16, 6)
    d = gen.c5_inputs(T, 4400, DEV)["c5_rmsnorm"]
    y = torch.zeros((T, 4096), dtype=torch.bfloat16, device=DEV)
    other = gen.randn((T * 4, 1024), 4401, DEV, "bf16")
    s = torch.zeros((T * 4, 1024), dtype=torch.bfloat16, device=DEV)
    add = single_op_program("add", 2, "bf16")
    norm = W.get_program("c5_rmsnorm")
    ins_a = [d[n] for n, _ in norm.inputs]
    ca = B.encode_for(ctx, H.program(norm), ins_a, [y])
    cb = B.encode_for(ctx, H.program(add), [y.view(T * 4, 1024), other], [s])
    st = B.dvm_stack_dependent([ca, cb], [-1, -1, -1, 2, -1, -1])
    ws = torch.zeros(B.WORKSPACE_BYTES // 4, dtype=torch.int32, device=DEV)
    ptrs = [t.data_ptr() for t in ins_a + [y, y, other, s]] + [ws.data_ptr()]
    stream = torch.cuda.current_stream().cuda_stream
    ctx.set_sync_limit(1)
    B.dvm_run(ctx, st, ptrs, stream)
    assert B.workspace_gave_up(ws.data_ptr(), stream)
    ctx.set_sync_limit(1 << 20)
    B.dvm_run(ctx, st, ptrs, stream)
    assert not B.workspace_gave_up(ws.data_ptr(), stream)
    want = (y.view(T * 4, 1024).float() + other.float()).to(torch.bfloat16)
    assert torch.equal(_bits(s), _bits(want))


def test_run_refuses_an_undeclared_dependence():
    say("dvm_stack of parts of which one reads what the other writes: refused by dvm_run")
    ctx = dep_ctx()
    T = 16
    d = gen.c5_inputs(T, 4500, DEV)["c5_rmsnorm"]
    norm = W.get_program("c5_rmsnorm")
    ins = [d[n] for n, _ in norm.inputs]
    y = torch.zeros((T, 4096), dtype=torch.bfloat16, device=DEV)
    z = torch.zeros((T, 4096), dtype=torch.bfloat16, device=DEV)
    ca = B.encode_for(ctx, H.program(norm), ins)
    st = B.dvm_stack([ca, ca])
    stream = torch.cuda.current_stream().cuda_stream
    with pytest.raises(B.DvmError) as e:
        B.dvm_run(ctx, st, [t.data_ptr() for t in ins + [y, y, ins[1], z]], stream)     # part 1 reads y
    assert e.value.status == -1
    with pytest.raises(B.DvmError):
        B.dvm_run(ctx, st, [t.data_ptr() for t in ins + [y] + ins + [y]], stream)       # both write y
    # declared as the same buffer but passed different pointers
    sd = B.dvm_stack_dependent([ca, ca], [-1, -1, -1, 2, 1, -1])
    with pytest.raises(B.DvmError):
        B.dvm_run(ctx, sd, [t.data_ptr() for t in ins + [y, z, ins[1], z]], stream)
    B.dvm_run(ctx, sd, [t.data_ptr() for t in ins + [y, y, ins[1], z]], stream)
    torch.cuda.synchronize()
    a1, _ = H.run_vm(norm, d, ctx=ctx)
    a2, _ = H.run_vm(norm, {norm.inputs[0][0]: a1["y"], norm.inputs[1][0]: ins[1]}, ctx=ctx)
    assert torch.equal(_bits(z), _bits(a2["y"]))
