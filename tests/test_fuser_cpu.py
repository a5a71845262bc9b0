"""Streaming fuser, host side (no GPU): on an encode-only context a flush encodes the buffered
operators without launching, which shows what was fused, what was elided and when the buffer ran."""
import re

import pytest

from paper_2603_24239_amd import binding as B


def _ctx():
    return B.Context(-1)


def test_chain_fuses_into_one_launch_and_released_values_never_reach_memory():
    f = B.Fuser(_ctx())
    x = f.tensor(0x1000, "f32", B.make_shape((64, 1000)))
    y = f.tensor(0x2000, "f32", B.make_shape((64, 1000)))
    t = f.op("muls", [x], "f32", 0x3000, imm=2.0)
    u = f.op("add", [t, y], "f32", 0x4000)
    f.release(t)                         # the framework dropped the temporary before anything ran
    assert f.stats() == {"ops": 2, "launches": 0, "flushes": 0, "elided": 0}
    f.flush()
    assert f.stats() == {"ops": 2, "launches": 1, "flushes": 1, "elided": 1}
    txt = f.last_code().disasm()
    assert len(re.findall(r"\bstore\b", txt)) == 1 and "mul" in txt and "add" in txt
    f.flush()                            # nothing buffered: no launch
    assert f.stats()["launches"] == 1
    # the result is now a plain tensor and feeds the next buffer
    v = f.op("tanh", [u], "f32", 0x5000)
    f.flush()
    assert f.stats()["launches"] == 2 and v != u


def test_unfusable_operator_cuts_the_buffer_and_the_pieces_share_a_launch():
    f = B.Fuser(_ctx())
    a = f.tensor(0x1000, "f32", B.make_shape((8, 128)))
    b = f.tensor(0x2000, "f32", B.make_shape((5, 77)))
    f.op("exp", [a], "f32", 0x3000)
    f.op("neg", [b], "f32", 0x4000)      # another iteration space: a second piece, nothing runs yet
    assert f.stats()["launches"] == 0 and f.stats()["flushes"] == 0
    f.flush()
    assert f.stats()["launches"] == 1
    txt = f.last_code().disasm()
    assert "vstack.t" in txt and txt.count("segment ") == 2 and "waits" not in txt


def test_a_piece_that_reads_an_earlier_piece_waits_for_it():
    f = B.Fuser(_ctx())
    a = f.tensor(0x1000, "f32", B.make_shape((40, 257)))
    b = f.tensor(0x2000, "f32", B.make_shape((7, 1000)))
    t = f.op("tanh", [a], "f32", 0x3000)
    f.op("sigmoid", [b], "f32", 0x4000)         # cut
    f.op("mul", [t, a], "f32", 0x5000)          # cut again; reads the first piece's result from its buffer
    f.release(t)                                # released, but a later piece reads it: it is written all the same
    f.flush()
    st = f.stats()
    assert st["launches"] == 1 and st["elided"] == 0
    txt = f.last_code().disasm()
    assert txt.count("segment ") == 3
    # same rows, same tiles: the third piece waits for its own workgroup's stores only, no workspace needed
    assert txt.count("waits for this workgroup's own stores") == 1 and "workspace" not in txt
    assert "same_buffer_as=1" in txt            # t: output of piece 0 (tensor 1), input of piece 2


def test_pieces_that_need_all_of_an_earlier_piece_wait_in_the_kernel_or_start_a_launch():
    def issue(f):
        x = f.tensor(0x10000, "f32", B.make_shape((64, 1024)))
        w = f.tensor(0x20000, "f32", B.make_shape((5, 77)))
        t = f.op("exp", [x], "f32", 0x30000)
        f.op("sum", [t], "f32", 0x38000)        # a reduction: this piece is tiled by rows
        f.op("neg", [w], "f32", 0x40000)        # cut
        f.op("tanh", [t], "f32", 0x50000)       # cut; element-wise over the flattened tensor: other tiles than the producer's
        f.flush()

    f = B.Fuser(_ctx())
    issue(f)
    # no workspace: still one program, whose third piece starts a kernel launch of its own behind the first two
    assert f.stats()["launches"] == 2 and f.stats()["flushes"] == 1
    txt = f.last_code().disasm()
    assert txt.count("segment ") == 3 and txt.count("a kernel launch of its own") == 1 and "workspace" not in txt
    f = B.Fuser(_ctx())
    f.set_workspace(0x7000000, B.WORKSPACE_BYTES)
    issue(f)
    assert f.stats()["launches"] == 1
    txt = f.last_code().disasm()
    assert "waits until every workgroup has finished" in txt and "workspace" in txt
    with pytest.raises(B.DvmError):
        f.set_workspace(0x7000010, B.WORKSPACE_BYTES)       # not 256-byte aligned
    with pytest.raises(B.DvmError):
        f.set_workspace(0x7000000, 8)


def test_reduction_and_its_consumers_share_a_launch():
    f = B.Fuser(_ctx())
    x = f.tensor(0x1000, "bf16", B.make_shape((300, 4096)))
    w = f.tensor(0x2000, "bf16", B.make_shape((4096,)))
    ms = f.op("meansq", [x], "f32", 0x3000)
    v = f.op("adds", [ms], "f32", 0x3100, imm=1e-6)
    r = f.op("rsqrt", [v], "f32", 0x3200)
    n = f.op("mul", [x, r], "bf16", 0x4000)
    y = f.op("mul", [n, w], "bf16", 0x5000)
    for t in (ms, v, r, n):
        f.release(t)
    f.flush()
    st = f.stats()
    assert st["launches"] == 1 and st["elided"] == 4
    txt = f.last_code().disasm()
    assert "red.sumsq" in txt and len(re.findall(r"\bstores?\b", txt)) == 1
    assert y >= 0


def test_errors_and_limits():
    f = B.Fuser(_ctx())
    a = f.tensor(0x1000, "f32", B.make_shape((8, 128)))
    b = f.tensor(0x2000, "f32", B.make_shape((8, 100)))
    with pytest.raises(B.DvmError):
        f.op("add", [a, b], "f32", 0x3000)           # shapes do not broadcast
    with pytest.raises(B.DvmError):
        f.op("neg", [12345], "f32", 0x3000)          # unknown value
    # a long chain: the buffer runs by itself when it is full
    cur = a
    for k in range(100):
        nxt = f.op("adds", [cur], "f32", 0x10000 + 0x1000 * k, imm=1.0)
        if cur != a:
            f.release(cur)
        cur = nxt
    f.flush()
    st = f.stats()
    assert st["ops"] == 100 and 2 <= st["launches"] <= 5 and st["elided"] >= 95


def test_reduction_along_the_penultimate_axis_and_its_epilogue_share_a_launch():
    f = B.Fuser(_ctx())
    x = f.tensor(0x1000, "f32", B.make_shape((6, 50, 300)))
    e = f.op("exp", [x], "f32", 0x2000)
    s = f.op("csum", [e], "f32", 0x3000)
    l = f.op("log", [s], "f32", 0x4000)          # on [6, 1, 300]: joins as the epilogue
    f.release(e)
    f.release(s)
    f.flush()
    assert f.stats() == {"ops": 3, "launches": 1, "flushes": 1, "elided": 2}
    txt = f.last_code().disasm()
    per_row, epilogue = txt.split("; epilogue")
    assert "exp" in per_row and "acc.sum" in per_row and "log" in epilogue and len(re.findall(r"store\b", txt)) == 1
    # a full-size operator on the reduced value cannot be part of that program: the group falls back to
    # one launch per operator
    e = f.op("exp", [x], "f32", 0x2000)
    s = f.op("csum", [e], "f32", 0x3000)
    d = f.op("sub", [x, s], "f32", 0x5000)
    f.flush()
    assert f.stats()["launches"] == 1 + 3
    # rank 1 has no penultimate axis
    v = f.tensor(0x6000, "f32", B.make_shape((64,)))
    with pytest.raises(B.DvmError):
        f.op("csum", [v], "f32", 0x7000)


def test_pieces_that_fit_no_common_interpreter_variant_run_one_by_one():
    f = B.Fuser(_ctx())
    f.set_workspace(0x7000000, B.WORKSPACE_BYTES)
    x = f.tensor(0x10000, "f32", B.make_shape((64, 1024)))
    w = f.tensor(0x20000, "f32", B.make_shape((5, 77)))
    t = f.op("exp", [x], "f32", 0x30000)
    f.op("neg", [w], "f32", 0x40000)
    f.op("csum", [t], "f32", 0x50000)   # its streaming form runs in the small-tile variants only, exp was planned for a larger one
    f.flush()
    assert f.stats()["launches"] == 3
