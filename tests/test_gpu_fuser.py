"""Streaming fuser on the GPU: operators issued one by one (the host decides the graph as it goes),
results compared with the oracle evaluating the same operator sequence."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2603_24239_amd import binding as B
from workloads import gen
from workloads import programs as W
from workloads.programs import _p

from . import harness as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[case] {msg}", flush=True)


def _fuser():
    return B.Fuser(H.gpu_ctx(), torch.cuda.current_stream().cuda_stream)


def test_if_else_add_stream_with_host_side_branches():
    """(a > b ? 2x : 4x) + y with the branch taken on the host (the paper's dynamic control-flow
    workload, Table 2): which multiply is issued differs from instance to instance."""
    f = _fuser()
    shapes = [sh for sh in gen.if_else_add_shapes(40) if sh[0] * sh[1] * sh[2] <= 2e7][:12]     # the oracle's share of the time
    for k, (b, s, ff, flag) in enumerate(shapes):
        say(f"if-else-add {k}: [{b},{s},{ff}] branch={flag}")
        x = gen.randn((b, s, ff), 800 + k, DEV)
        y = gen.randn((b, s, ff), 900 + k, DEV)
        tmp = torch.empty_like(x)
        out = torch.full_like(x, float("nan"))
        vx = f.tensor(x.data_ptr(), "f32", B.shape_of_tensor(x))
        vy = f.tensor(y.data_ptr(), "f32", B.shape_of_tensor(y))
        t = f.op("muls", [vx], "f32", tmp.data_ptr(), imm=2.0 if flag else 4.0)
        o = f.op("add", [t, vy], "f32", out.data_ptr())
        f.release(t)
        f.flush()
        torch.cuda.synchronize()
        desc = W.get_program("if_else_add_true" if flag else "if_else_add_false")
        rounded, exact = H.run_oracle(desc, {"x": x, "y": y})
        name = desc.outputs[0][0]
        H.compare(out, rounded[name], exact[name], "f32", False, f"if-else-add {k}")
        for v in (vx, vy, o):
            f.release(v)
    st = f.stats()
    assert st["launches"] == len(shapes) and st["elided"] == len(shapes)


def test_rmsnorm_issued_op_by_op_equals_the_fused_program():
    f = _fuser()
    d = gen.c2_inputs(3, 333, 77, DEV)
    x, w = d["x"], d["w"]
    rows = torch.empty((3, 333, 1), dtype=torch.float32, device=DEV)
    rows2, rows3 = torch.empty_like(rows), torch.empty_like(rows)
    n = torch.empty_like(x)
    y = torch.full_like(x, float("nan"))
    vx = f.tensor(x.data_ptr(), "bf16", B.shape_of_tensor(x))
    vw = f.tensor(w.data_ptr(), "bf16", B.shape_of_tensor(w))
    ms = f.op("meansq", [vx], "f32", rows.data_ptr())
    v = f.op("adds", [ms], "f32", rows2.data_ptr(), imm=1e-6)
    r = f.op("rsqrt", [v], "f32", rows3.data_ptr())
    nn_ = f.op("mul", [vx, r], "bf16", n.data_ptr())
    f.op("mul", [nn_, vw], "bf16", y.data_ptr())
    for t in (ms, v, nn_):
        f.release(t)                    # r stays referenced: it must be written as a second output
    f.flush()
    torch.cuda.synchronize()
    assert f.stats()["launches"] == 1
    desc = W.get_program("c2_rmsnorm_basic")
    rounded, exact = H.run_oracle(desc, {"x": x, "w": w})
    H.compare(y, rounded["y"], exact["y"], "bf16", True, "fuser rmsnorm")
    # the kept row value against the oracle's intermediate
    keep = _p("keep_r", [("x", "bf16")], [("ms", "meansq", ["x"], {}), ("v", "adds", ["ms"], {"imm": 1e-6}),
                                          ("r", "rsqrt", ["v"], {})], [("r", "f32")])
    rr, re_ = H.run_oracle(keep, {"x": x})
    H.compare(rows3, rr["r"], re_["r"], "f32", True, "fuser kept row value")


def test_pieces_of_different_shapes_run_in_order_in_one_launch():
    f = _fuser()
    a = gen.randn((40, 257), 61, DEV)
    b = gen.randn((7, 1000), 62, DEV)
    ea, eb, sa = torch.empty_like(a), torch.empty_like(b), torch.empty_like(a)
    va = f.tensor(a.data_ptr(), "f32", B.shape_of_tensor(a))
    vb = f.tensor(b.data_ptr(), "f32", B.shape_of_tensor(b))
    t = f.op("tanh", [va], "f32", ea.data_ptr())
    f.op("sigmoid", [vb], "f32", eb.data_ptr())          # does not fuse with the first: a second piece
    f.op("mul", [t, va], "f32", sa.data_ptr())           # a third piece; reads the first one's result from its buffer
    f.flush()
    torch.cuda.synchronize()
    assert f.stats()["launches"] == 1                    # cut-and-stack: the three pieces are one launch
    assert f.last_code().disasm().count("segment ") == 3
    # the oracle evaluates the same three operators
    pa = _p("tanh_then_mul", [("a", "f32")], [("t", "tanh", ["a"], {}), ("m", "mul", ["t", "a"], {})], [("t", "f32"), ("m", "f32")])
    pb = _p("sigmoid_b", [("b", "f32")], [("s", "sigmoid", ["b"], {})], [("s", "f32")])
    ra, xa = H.run_oracle(pa, {"a": a})
    rb, xb = H.run_oracle(pb, {"b": b})
    H.compare(ea, ra["t"], xa["t"], "f32", False, "fuser tanh")
    H.compare(sa, ra["m"], xa["m"], "f32", False, "fuser tanh * a")
    H.compare(eb, rb["s"], xb["s"], "f32", False, "fuser sigmoid")


def test_reduction_along_the_penultimate_axis_joins_the_buffer():
    # exp, column sum and the log of the sums arrive one by one and run as one launch; a full-size op on
    # the reduced value cannot join that launch's program and runs after it
    say("fuser: exp -> csum -> log, then x - logsumexp")
    f = _fuser()
    x = gen.randn((6, 50, 300), 2100, DEV)
    e = torch.empty_like(x)
    s_ = torch.empty((6, 1, 300), dtype=torch.float32, device=DEV)
    l = torch.full((6, 1, 300), float("nan"), dtype=torch.float32, device=DEV)
    d = torch.full_like(x, float("nan"))
    vx = f.tensor(x.data_ptr(), "f32", B.shape_of_tensor(x))
    ve = f.op("exp", [vx], "f32", e.data_ptr())
    vs = f.op("csum", [ve], "f32", s_.data_ptr())
    vl = f.op("log", [vs], "f32", l.data_ptr())
    f.release(ve)
    f.release(vs)
    vd = f.op("sub", [vx, vl], "f32", d.data_ptr())
    f.flush()
    torch.cuda.synchronize()
    st = f.stats()
    assert st["ops"] == 4 and st["launches"] >= 2, st
    # the oracle evaluates the same four operators
    prog = _p("col_logsumexp", [("x", "f32")],
              [("e", "exp", ["x"], {}), ("s", "csum", ["e"], {}), ("l", "log", ["s"], {}), ("d", "sub", ["x", "l"], {})],
              [("l", "f32"), ("d", "f32")])
    rounded, exact = H.run_oracle(prog, {"x": x})
    H.compare(l, rounded["l"], exact["l"], "f32", True, "fuser logsumexp over columns")
    H.compare(d, rounded["d"], exact["d"], "f32", True, "fuser x - logsumexp")
    for v in (vx, vl, vd):
        f.release(v)


def test_pieces_with_a_grid_wide_dependence_use_the_workspace():
    say("fuser: exp + row sum | neg (other shape) | tanh of the first piece's result over other tiles, one launch with workspace")
    f = _fuser()
    ws = torch.empty(B.WORKSPACE_BYTES // 4, dtype=torch.int32, device=DEV)
    f.set_workspace(ws.data_ptr(), B.WORKSPACE_BYTES)
    x = gen.randn((700, 1540), 2200, DEV)
    w = gen.randn((5, 77), 2201, DEV)
    e = torch.full_like(x, float("nan"))
    th = torch.full_like(x, float("nan"))
    n = torch.full_like(w, float("nan"))
    s_ = torch.full((700, 1), float("nan"), dtype=torch.float32, device=DEV)
    vx = f.tensor(x.data_ptr(), "f32", B.shape_of_tensor(x))
    vw = f.tensor(w.data_ptr(), "f32", B.shape_of_tensor(w))
    ve = f.op("exp", [vx], "f32", e.data_ptr())
    f.op("sum", [ve], "f32", s_.data_ptr())
    f.op("neg", [vw], "f32", n.data_ptr())
    f.op("tanh", [ve], "f32", th.data_ptr())
    f.release(ve)
    f.flush()
    assert not B.workspace_gave_up(ws.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert f.stats()["launches"] == 1 and "waits until every workgroup" in f.last_code().disasm()
    pe = _p("exp_sum_tanh", [("x", "f32")], [("e", "exp", ["x"], {}), ("s", "sum", ["e"], {}), ("t", "tanh", ["e"], {})],
            [("e", "f32"), ("s", "f32"), ("t", "f32")])
    r, xct = H.run_oracle(pe, {"x": x})
    H.compare(e, r["e"], xct["e"], "f32", False, "fuser exp")
    H.compare(s_, r["s"], xct["s"], "f32", True, "fuser row sum of exp")
    H.compare(th, r["t"], xct["t"], "f32", False, "fuser tanh of exp")
    pn = _p("neg_w", [("w", "f32")], [("n", "neg", ["w"], {})], [("n", "f32")])
    r, xct = H.run_oracle(pn, {"w": w})
    H.compare(n, r["n"], xct["n"], "f32", False, "fuser neg")


def test_pieces_without_a_common_variant_fall_back_to_launches_in_order():
    say("fuser: exp | neg | column sum of exp: no interpreter variant holds all three, launched one by one")
    f = _fuser()
    x = gen.randn((3, 700, 520), 2300, DEV)
    w = gen.randn((5, 77), 2301, DEV)
    e = torch.full_like(x, float("nan"))
    n = torch.full_like(w, float("nan"))
    s_ = torch.full((3, 1, 520), float("nan"), dtype=torch.float32, device=DEV)
    vx = f.tensor(x.data_ptr(), "f32", B.shape_of_tensor(x))
    vw = f.tensor(w.data_ptr(), "f32", B.shape_of_tensor(w))
    ve = f.op("exp", [vx], "f32", e.data_ptr())
    f.op("neg", [vw], "f32", n.data_ptr())
    f.op("csum", [ve], "f32", s_.data_ptr())
    f.release(ve)
    f.flush()
    torch.cuda.synchronize()
    pe = _p("exp_then_csum", [("x", "f32")], [("e", "exp", ["x"], {}), ("s", "csum", ["e"], {})], [("e", "f32"), ("s", "f32")])
    r, xct = H.run_oracle(pe, {"x": x})
    H.compare(e, r["e"], xct["e"], "f32", False, "fuser exp")
    H.compare(s_, r["s"], xct["s"], "f32", True, "fuser column sum of exp")
    assert torch.equal(n, -w)
