"""Parity at the full sizes of the benchmark configurations, in the launch configuration bench.py times.

The oracle cannot evaluate multi-gigabyte instances in seconds, but every program on the path is
independent per row of the reduced (last) axis, so the oracle evaluates a seeded sample of rows
(the first and last rows always among them) and the HIP result is compared on exactly those rows,
element by element, to the same tolerance as the small cases.
"""
from __future__ import annotations

import numpy as np
import pytest
import torch

from workloads import gen
from workloads import programs as W

from . import harness as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[case] {msg}", flush=True)


def sample_rows(n_rows: int, k: int, seed: int) -> torch.Tensor:
    rng = np.random.default_rng(seed)
    pick = set(rng.integers(0, n_rows, size=min(k, n_rows)).tolist()) | {0, n_rows - 1}
    return torch.tensor(sorted(pick), dtype=torch.long)


def check_rows(desc, ins_rows, outs_rows, what):
    rounded, exact = H.run_oracle(desc, ins_rows)
    red = H.has_reduction(desc)
    worst = 0.0
    for n, dt in desc.outputs:
        worst = max(worst, H.compare(outs_rows[n], rounded[n], exact[n], dt, red, f"{what}:{n}"))
    return worst


def test_c2_rmsnorm_largest_instance():
    shapes = gen.c2_shapes()
    B, S = max(shapes, key=lambda bs: bs[0] * bs[1])
    say(f"c2 rmsnorm full size B={B} S={S}")
    d = gen.c2_inputs(B, S, gen.BASE_SEED + 2999, DEV)
    desc = W.get_program("c2_rmsnorm")
    outs, code = H.run_vm(desc, d)
    y = outs["y"].reshape(B * S, 4096)
    x = d["x"].reshape(B * S, 4096)
    rows = sample_rows(B * S, 192, 1).to(DEV)
    check_rows(desc, {"x": x[rows], "w": d["w"]}, {"y": y[rows]}, "c2 full")


def test_c4_chain_largest_instance():
    T = max(gen.c4_shapes())
    say(f"c4 chain full size T={T}")
    d = gen.c4_inputs(T, gen.BASE_SEED + 4999, DEV)
    desc = W.get_program("c4_chain")
    outs, code = H.run_vm(desc, d)
    rows = sample_rows(T, 96, 2).to(DEV)
    ins = {k: (v[rows] if v.dim() == 2 else v) for k, v in d.items()}
    check_rows(desc, ins, {"y": outs["y"][rows]}, "c4 full")


def test_c3_masked_softmax_large_instance():
    # the largest S of the stream with B = 1: 32 * S rows of S fp32 scores (about 2 GiB in, 2 GiB out)
    S = max(s for _, s in gen.c3_shapes())
    say(f"c3 masked softmax full size B=1 S={S}")
    d = gen.c3_inputs(1, S, gen.BASE_SEED + 3999, DEV)
    desc = W.get_program("c3_masked_softmax")
    outs, code = H.run_vm(desc, d)
    out_name = desc.outputs[0][0]
    p = outs[out_name].reshape(32 * S, S)
    z = d["z"].reshape(32 * S, S)
    rows = sample_rows(32 * S, 128, 3).to(DEV)
    mrows = d["mask"][rows % S]
    check_rows(desc, {"z": z[rows], "mask": mrows}, {out_name: p[rows]}, "c3 full")
    # masked positions are exactly zero, every row sums to one
    assert torch.all(p[rows][mrows == float("-inf")] == 0)
    assert torch.allclose(p[rows].sum(-1), torch.ones(len(rows), device=DEV), atol=1e-5)
    del outs, d, p, z
    torch.cuda.empty_cache()


def test_c5_layer_at_max_tokens():
    T = 8192
    say(f"c5 programs full size T={T}")
    d = gen.c5_inputs(T, gen.BASE_SEED + 5999, DEV)
    rows = sample_rows(T, 48, 4).to(DEV)
    for name, key in [("c5_rmsnorm", "c5_rmsnorm"), ("c5_residual", "c5_residual_a"), ("c5_silu_gate", "c5_silu_gate")]:
        desc = W.get_program(name)
        outs, _ = H.run_vm(desc, d[key])
        ins = {k: (v[rows] if v.dim() == 2 else v) for k, v in d[key].items()}
        check_rows(desc, ins, {n: outs[n][rows] for n, _ in desc.outputs}, f"c5 full {name}")
        del outs
    say("c5 rope full size (views)")
    desc = W.get_program("c5_rope")
    out = torch.full((T, 32, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    views = {"y1": out[..., :64], "y2": out[..., 64:]}
    H.run_vm(desc, d["c5_rope"], views)
    assert not torch.isnan(out.float()).any()
    ins = {k: v[rows] for k, v in d["c5_rope"].items()}
    check_rows(desc, ins, {"y1": out[rows][..., :64], "y2": out[rows][..., 64:]}, "c5 full rope")
    del out
    say("c5 softmax full size [32, T, T//8+1]")
    desc = W.get_program("c5_softmax")
    z = d["c5_softmax"]["z"]
    outs, _ = H.run_vm(desc, {"z": z})
    L = T // 8 + 1
    out_name = desc.outputs[0][0]
    r2 = sample_rows(32 * T, 96, 5).to(DEV)
    check_rows(desc, {"z": z.reshape(32 * T, L)[r2]}, {out_name: outs[out_name].reshape(32 * T, L)[r2]}, "c5 full softmax")
    del outs, d
    torch.cuda.empty_cache()


# ---- every row of one instance per configuration in which a workgroup runs several tiles -------------------------
# (the oracle goes over the instance in blocks of rows; the instance is sized so that this takes seconds)

def check_every_row(desc, make_block_inputs, outs2d, n_rows, what, block=2048):
    red = H.has_reduction(desc)
    worst = 0.0
    for lo in range(0, n_rows, block):
        hi = min(n_rows, lo + block)
        rounded, exact = H.run_oracle(desc, make_block_inputs(lo, hi))
        for n, dt in desc.outputs:
            worst = max(worst, H.compare(outs2d[n][lo:hi], rounded[n], exact[n], dt, red, f"{what} rows {lo}..{hi}:{n}"))
    return worst


def _tiles_per_workgroup(code):
    inf = code.info()
    return inf.n_tiles / max(1, inf.grid)


def test_c2_every_row_of_a_multi_tile_instance():
    B, S = 4, 2048
    say(f"c2 rmsnorm, every row, B={B} S={S}")
    d = gen.c2_inputs(B, S, gen.BASE_SEED + 2777, DEV)
    desc = W.get_program("c2_rmsnorm")
    outs, code = H.run_vm(desc, d)
    assert _tiles_per_workgroup(code) >= 2
    x = d["x"].reshape(B * S, 4096)
    check_every_row(desc, lambda lo, hi: {"x": x[lo:hi], "w": d["w"]}, {"y": outs["y"].reshape(B * S, 4096)}, B * S, "c2 every row")


def test_c4_every_row_of_a_multi_tile_instance():
    T = 3100
    say(f"c4 chain, every row, T={T}")
    d = gen.c4_inputs(T, gen.BASE_SEED + 4777, DEV)
    desc = W.get_program("c4_chain")
    outs, code = H.run_vm(desc, d)
    assert _tiles_per_workgroup(code) >= 2
    check_every_row(desc, lambda lo, hi: {k: (v[lo:hi] if v.dim() == 2 else v) for k, v in d.items()}, {"y": outs["y"]}, T, "c4 every row",
                    block=1024)


def test_c3_every_row_of_a_multi_tile_instance():
    S = 701                                     # (rows that are not whole lines: the blocked assignment with a pinned mask row)
    say(f"c3 masked softmax, every row, B=2 S={S}")
    d = gen.c3_inputs(2, S, gen.BASE_SEED + 3777, DEV)
    desc = W.get_program("c3_masked_softmax")
    outs, code = H.run_vm(desc, d)
    assert _tiles_per_workgroup(code) >= 2
    out_name = desc.outputs[0][0]
    n_rows = 2 * 32 * S
    z = d["z"].reshape(n_rows, S)
    idx = torch.arange(n_rows, device=DEV) % S
    check_every_row(desc, lambda lo, hi: {"z": z[lo:hi], "mask": d["mask"][idx[lo:hi]]}, {out_name: outs[out_name].reshape(n_rows, S)},
                    n_rows, "c3 every row", block=8192)


def test_c5_every_row_of_a_layer():
    T = 1500
    say(f"c5 programs, every row, T={T}")
    d = gen.c5_inputs(T, gen.BASE_SEED + 5777, DEV)
    for name, key in [("c5_rmsnorm", "c5_rmsnorm"), ("c5_residual", "c5_residual_a"), ("c5_silu_gate", "c5_silu_gate")]:
        desc = W.get_program(name)
        outs, _ = H.run_vm(desc, d[key])
        check_every_row(desc, lambda lo, hi: {k: (v[lo:hi] if v.dim() == 2 else v) for k, v in d[key].items()},
                        {n: outs[n] for n, _ in desc.outputs}, T, f"c5 every row {name}")
    desc = W.get_program("c5_rope")
    out = torch.full((T, 32, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    H.run_vm(desc, d["c5_rope"], {"y1": out[..., :64], "y2": out[..., 64:]})
    check_every_row(desc, lambda lo, hi: {k: v[lo:hi] for k, v in d["c5_rope"].items()}, {"y1": out[..., :64], "y2": out[..., 64:]}, T,
                    "c5 every row rope", block=512)
    desc = W.get_program("c5_softmax")
    T = 2500            # (scores of a longer step: enough rows that a workgroup runs several tiles)
    z = gen.randn((32, T, T // 8 + 1), gen.BASE_SEED + 5778, DEV, "bf16")
    L = T // 8 + 1
    outs, code = H.run_vm(desc, {"z": z})
    assert _tiles_per_workgroup(code) >= 2
    out_name = desc.outputs[0][0]
    check_every_row(desc, lambda lo, hi: {"z": z.reshape(32 * T, L)[lo:hi]}, {out_name: outs[out_name].reshape(32 * T, L)}, 32 * T,
                    "c5 every row softmax", block=16384)
