"""dvm_run_batched on the GPU: one launch runs a program (or a stack of programs) over several sets of tensors.
Every set must come out with exactly the bits a launch of its own gives, and match the oracle."""
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


def _table(n_sets, n_tensors):
    return torch.empty(n_sets * n_tensors, dtype=torch.int64, device=DEV)


def _outputs(desc, code):
    return [torch.zeros(s, dtype=H._TORCH_DT[dt], device=DEV) for (_, dt), s in zip(desc.outputs, code.out_shapes)]


@pytest.mark.parametrize("name,make", [
    ("c2_rmsnorm", lambda k: gen.c2_inputs(2, 300 + 7 * k - 7 * k, 7000 + k, DEV)),
    ("c4_chain", lambda k: gen.c4_inputs(77, 7100 + k, DEV)),          # (keeps weight vectors in LDS: the prologue runs per set)
    ("c3_masked_softmax", lambda k: gen.c3_inputs(1, 130, 7200 + k, DEV)),
])
def test_one_program_over_several_sets(name, make):
    say(f"batched: {name} over 5 sets")
    ctx = H.gpu_ctx()
    desc = W.get_program(name)
    prog = H.program(desc)
    stream = torch.cuda.current_stream().cuda_stream
    sets_in = [[make(k)[n] for n, _ in desc.inputs] for k in range(5)]
    code = B.encode_for(ctx, prog, sets_in[0])
    outs_b = [_outputs(desc, code) for _ in range(5)]
    outs_1 = [_outputs(desc, code) for _ in range(5)]
    n_t = len(sets_in[0]) + len(outs_b[0])
    table = _table(5, n_t)
    B.dvm_run_batched(ctx, code, [[t.data_ptr() for t in i + o] for i, o in zip(sets_in, outs_b)], table.data_ptr(), table.numel() * 8, stream)
    for i, o in zip(sets_in, outs_1):
        B.dvm_run(ctx, code, [t.data_ptr() for t in i + o], stream)
    torch.cuda.synchronize()
    for k in range(5):
        for (n, dt), got, alone in zip(desc.outputs, outs_b[k], outs_1[k]):
            assert torch.equal(_bits(got), _bits(alone)), f"{name} set {k}: {n} differs from a launch of its own"
    ins = {n: t for (n, _), t in zip(desc.inputs, sets_in[3])}
    rounded, exact = H.run_oracle(desc, ins)
    for (n, dt), got in zip(desc.outputs, outs_b[3]):
        H.compare(got, rounded[n], exact[n], dt, H.has_reduction(desc), f"batched {name} set 3: {n}")


@pytest.mark.parametrize("limits,copies,T", [((16, 6), 1, 45), ((32, 2), 32, 45), ((32, 2), 32, 300), ((16, 4), 8, 131)])
def test_a_stack_of_programs_over_several_sets(limits, copies, T):
    say(f"batched: the six programs of a layer, stacked, over 4 sets (T={T}, variant limits {limits}, planned for {copies} copies in flight)")
    ctx = B.Context(torch.cuda.current_device())
    ctx.set_limits(*limits)
    ctx.set_copies_in_flight(copies)
    stream = torch.cuda.current_stream().cuda_stream
    names = ["c5_rmsnorm", "c5_rope", "c5_softmax", "c5_residual", "c5_silu_gate", "c5_residual"]
    keys = ["c5_rmsnorm", "c5_rope", "c5_softmax", "c5_residual_a", "c5_silu_gate", "c5_residual_b"]

    def layer(seed):
        d = gen.c5_inputs(T, seed, DEV)
        rope_out = torch.zeros((T, 32, 128), dtype=torch.bfloat16, device=DEV)
        codes, tensors, outs = [], [], []
        for nm, key in zip(names, keys):
            desc = W.get_program(nm)
            ins = [d[key][n] for n, _ in desc.inputs]
            if nm == "c5_rope":
                o = [rope_out[..., :64], rope_out[..., 64:]]
                code = B.encode_for(ctx, H.program(desc), ins, o)
            else:
                code = B.encode_for(ctx, H.program(desc), ins)
                o = _outputs(desc, code)
            codes.append(code)
            tensors += ins + o
            outs.append(o if nm != "c5_rope" else [rope_out])
        return codes, tensors, outs, d

    layers_b = [layer(7300 + k) for k in range(4)]
    layers_1 = [layer(7300 + k) for k in range(4)]
    st = B.dvm_stack(layers_b[0][0])
    n_t = len(layers_b[0][1])
    table = _table(4, n_t)
    B.dvm_run_batched(ctx, st, [[t.data_ptr() for t in L[1]] for L in layers_b], table.data_ptr(), table.numel() * 8, stream)
    for L in layers_1:
        B.dvm_run(ctx, st, [t.data_ptr() for t in L[1]], stream)
    torch.cuda.synchronize()
    for k in range(4):
        for ob, o1 in zip(layers_b[k][2], layers_1[k][2]):
            for a, b in zip(ob, o1):
                assert torch.equal(_bits(a), _bits(b)), f"set {k}: a stacked part differs from the launch of its own"
    assert float(layers_b[2][2][0][0].float().abs().max()) > 0      # (the outputs were written at all)
    # one set against the oracle, program by program
    d = layers_b[1][3]
    for nm, key, o in zip(names, keys, layers_b[1][2]):
        desc = W.get_program(nm)
        rounded, exact = H.run_oracle(desc, d[key])
        got = {"y1": o[0][..., :64], "y2": o[0][..., 64:]} if nm == "c5_rope" else {n: t for (n, _), t in zip(desc.outputs, o)}
        for n, dt in desc.outputs:
            H.compare(got[n], rounded[n], exact[n], dt, H.has_reduction(desc), f"batched layer, {nm}: {n}")


def test_argument_errors():
    ctx = H.gpu_ctx()
    desc = W.get_program("c2_rmsnorm")
    d = gen.c2_inputs(1, 8, 7400, DEV)
    ins = [d[n] for n, _ in desc.inputs]
    code = B.encode_for(ctx, H.program(desc), ins)
    out = _outputs(desc, code)
    ptrs = [t.data_ptr() for t in ins + out]
    table = _table(2, 3)
    stream = torch.cuda.current_stream().cuda_stream
    with pytest.raises(B.DvmError):
        B.dvm_run_batched(ctx, code, [ptrs, ptrs], table.data_ptr(), 8, stream)             # table too small
    with pytest.raises(B.DvmError):
        B.dvm_run_batched(ctx, code, [ptrs, [ptrs[0], 0, ptrs[2]]], table.data_ptr(), 48, stream)   # null pointer in the second set
    with pytest.raises(B.DvmError):
        B.dvm_run_batched(ctx, code, [ptrs, ptrs], table.data_ptr() + 4, 48, stream)        # misaligned table
    B.dvm_run_batched(ctx, code, [ptrs, ptrs], table.data_ptr(), 48, stream)                # (both sets write the same output)
    torch.cuda.synchronize()
    alone, _ = H.run_vm(desc, d)
    assert torch.equal(_bits(out[0]), _bits(alone[desc.outputs[0][0]]))
