"""Differential test: seeded random operator programs (elementwise chains, broadcasts, row reductions
and their consumers, selects, strided inputs) on the HIP VM against the oracle, element by element."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2603_24239_amd import binding as B
from workloads import gen

from . import harness as H
from . import random_programs as R

pytestmark = pytest.mark.gpu
DEV = "cuda"
_DT = {"f32": torch.float32, "bf16": torch.bfloat16}


def _tensor(shape, dt, layout, seed):
    """A tensor of the given logical shape whose storage follows `layout`."""
    shape = tuple(shape)
    strides = R.layout_of(shape, layout)
    n_store = 1 + sum((s - 1) * st for s, st in zip(shape, strides)) if all(s > 0 for s in shape) else 0
    base = gen.randn((max(n_store, 1),), seed, DEV, dt)
    return torch.as_strided(base, shape, strides)


def _run(seed, ctx=None):
    desc, specs, dom, has_red = R.make(seed)
    ins = {n: _tensor(specs[n][0], specs[n][1], specs[n][2], 7000 + 13 * seed + i) for i, (n, _) in enumerate(desc.inputs)}
    print(f"[case] seed {seed}: dominant shape {dom}, {len(desc.ops)} ops, inputs "
          f"{[(tuple(t.shape), str(t.dtype)[6:], specs[n][2]) for n, t in ins.items()]}", flush=True)
    try:
        outs, code = H.run_vm(desc, ins, ctx=ctx)
    except B.DvmError as e:
        assert e.status in (-5, -4), str(e)
        return False
    rounded, exact = H.run_oracle(desc, ins)
    for n, dt in desc.outputs:
        H.compare(outs[n], rounded[n], exact[n], dt, has_red, f"seed {seed}:{n}")
    return True


@pytest.mark.parametrize("block", range(8))
def test_random_programs_match_the_oracle(block):
    ran = sum(_run(seed) for seed in range(block * 20, block * 20 + 20))
    assert ran >= 14, "too many programs refused for the test to mean anything"


def test_random_programs_under_stacking_limits():
    ctx = B.Context(torch.cuda.current_device())
    ctx.set_limits(16, 4)
    ran = sum(_run(seed, ctx) for seed in range(200, 240))
    assert ran >= 28


def test_random_programs_planned_for_wide_tiles_and_a_shared_launch():
    """The same differential test under the planner settings of a batched run: 64 elements per lane allowed, the cost
    model told that 32 copies of every program share the launch."""
    ctx = B.Context(torch.cuda.current_device())
    ctx.set_limits(64, 6)
    ctx.set_copies_in_flight(32)
    ran = sum(_run(seed, ctx) for seed in range(300, 340))
    assert ran >= 28
