"""Host-side tests (no GPU) of temporal stacking of dependent parts (Section 5.1: stacking does not require
independent operators): which synchronisation point a part gets, the workspace entry, the validator, errors."""
import re

import pytest

from paper_2603_24239_amd import binding as B
from workloads import programs as W
from workloads.programs import _p, single_op_program


@pytest.fixture(scope="module")
def ctx():
    c = B.Context(-1)
    c.set_limits(16, 6)
    return c


def _rmsnorm(ctx, T):
    return B.dvm_encode(ctx, B.Program(W.get_program("c5_rmsnorm")), [B.make_shape((T, 4096)), B.make_shape((4096,))])


def _segments(code):
    return [l for l in code.disasm().splitlines() if l.startswith("segment ") or l.lstrip().startswith("; waits")]


def test_consumer_with_the_same_rows_waits_for_its_own_workgroup_only(ctx):
    T = 3000
    a = _rmsnorm(ctx, T)                                    # x, w -> y
    soft = _p("soft_bf16", [("z", "bf16")], [("y", "softmax", ["z"], {})], [("y", "bf16")])
    b = B.dvm_encode(ctx, B.Program(soft), [B.make_shape((T, 4096))])     # z -> p, z is a's y
    st = B.dvm_stack_dependent([a, b], [-1, -1, -1, 2, -1])
    st.validate()
    txt = st.disasm()
    assert txt.count("waits for this workgroup's own stores") == 1
    assert "every workgroup" not in txt
    assert not st.needs_workspace() and st.info().n_tensors == 5
    assert "same_buffer_as=2" in txt
    # the wait sits on the consumer, not on the producer
    seg = _segments(st)
    assert seg[0].startswith("segment 0") and seg[1].startswith("segment 1") and "waits" in seg[2]


def test_consumer_with_other_tiles_waits_for_the_whole_grid(ctx):
    T = 3000
    a = _rmsnorm(ctx, T)
    # an element-wise program over the same values seen as [T*4, 1024]: other rows per tile, other tiles
    add = single_op_program("add", 2, "bf16")
    b = B.dvm_encode(ctx, B.Program(add), [B.make_shape((T * 4, 1024)), B.make_shape((T * 4, 1024))])
    st = B.dvm_stack_dependent([a, b], [-1, -1, -1, 2, -1, -1])
    st.validate()
    txt = st.disasm()
    assert txt.count("waits until every workgroup has finished") == 1
    assert st.needs_workspace() and st.info().n_tensors == 7
    need, is_out, dt, al = st.tensor(6)
    assert need == B.WORKSPACE_BYTES and al == 256
    assert re.search(r"tensor 6: f32 workspace", txt)


def test_write_after_read_is_a_dependence_too(ctx):
    T = 500
    a = _rmsnorm(ctx, T)
    b = _rmsnorm(ctx, T)          # b writes the buffer a read as x
    st = B.dvm_stack_dependent([a, b], [-1, -1, -1, -1, -1, 0])
    assert "waits" in st.disasm()
    # both parts only read a shared input: no wait, no workspace, and nothing but the alias note differs from dvm_stack
    st2 = B.dvm_stack_dependent([a, b], [-1, -1, -1, -1, 1, -1])
    assert "waits" not in st2.disasm() and not st2.needs_workspace()
    assert B.dvm_stack_dependent([a, b], [-1] * 6).raw == B.dvm_stack([a, b]).raw


def test_three_parts_chain(ctx):
    T = 64
    a = _rmsnorm(ctx, T)
    b = _rmsnorm(ctx, T)
    c = _rmsnorm(ctx, T)
    # y_a -> x_b, y_b -> x_c, all share w
    st = B.dvm_stack_dependent([a, b, c], [-1, -1, -1, 2, 1, -1, 5, 1, -1])
    st.validate()
    assert st.disasm().count("waits for this workgroup's own stores") == 2


def test_argument_errors(ctx):
    a = _rmsnorm(ctx, 10)
    b = _rmsnorm(ctx, 10)
    with pytest.raises(B.DvmError) as e:
        B.dvm_stack_dependent([a, b], [-1, -1, -1, 2, -1])          # one entry short
    assert e.value.status == -1
    with pytest.raises(B.DvmError) as e:
        B.dvm_stack_dependent([a, b], [-1, -1, -1, 4, -1, -1])      # names a later entry
    assert e.value.status == -1
    f32 = B.dvm_encode(ctx, B.Program(single_op_program("exp", 1)), [B.make_shape((10, 4096))])
    with pytest.raises(B.DvmError) as e:
        B.dvm_stack_dependent([a, f32], [-1, -1, -1, 2, -1])        # bf16 buffer read as f32
    assert e.value.status == -4
    # a dependent stack is not a part of another one
    add = single_op_program("add", 2, "bf16")
    g = B.dvm_encode(ctx, B.Program(add), [B.make_shape((40, 1024)), B.make_shape((40, 1024))])
    st = B.dvm_stack_dependent([a, g], [-1, -1, -1, 2, -1, -1])
    assert st.needs_workspace()
    with pytest.raises(B.DvmError) as e:
        B.dvm_stack_dependent([st, a], [-1] * 10)
    assert e.value.status == -5


def test_validator_rejects_tampered_synchronisation(ctx):
    import struct
    T = 3000
    a = _rmsnorm(ctx, T)
    add = single_op_program("add", 2, "bf16")
    b = B.dvm_encode(ctx, B.Program(add), [B.make_shape((T * 4, 1024)), B.make_shape((T * 4, 1024))])
    st = B.dvm_stack_dependent([a, b], [-1, -1, -1, 2, -1, -1])
    words = list(struct.unpack("<%dI" % (len(st.raw) // 4), st.raw))
    # drop the workspace flag from the last tensor: a grid-wide wait without workspace must not validate
    ws_info = 8 + 6 * 3
    assert words[ws_info] & (1 << 9)
    bad = list(words)
    bad[ws_info] &= ~(1 << 9)
    with pytest.raises(B.DvmError):
        B.Bytecode(struct.pack("<%dI" % len(bad), *bad), []).validate()
    # a tensor that names a later entry as the same buffer
    bad = list(words)
    bad[8] |= 5 << 24
    with pytest.raises(B.DvmError):
        B.Bytecode(struct.pack("<%dI" % len(bad), *bad), []).validate()
    # a synchronisation flag in a plain meta-kernel
    words_a = list(struct.unpack("<%dI" % (len(a.raw) // 4), a.raw))
    flags_at = 8 + 3 * 3 + 20       # S_FLAGS of the only segment
    words_a[flags_at] |= 16
    with pytest.raises(B.DvmError):
        B.Bytecode(struct.pack("<%dI" % len(words_a), *words_a), []).validate()


def test_order_by_launch_needs_no_workspace(ctx):
    T = 3000
    a = _rmsnorm(ctx, T)
    add = single_op_program("add", 2, "bf16")
    b = B.dvm_encode(ctx, B.Program(add), [B.make_shape((T * 4, 1024)), B.make_shape((T * 4, 1024))])
    st = B.dvm_stack_dependent([a, b], [-1, -1, -1, 2, -1, -1], order_by="launch")
    st.validate()
    txt = st.disasm()
    assert txt.count("a kernel launch of its own") == 1 and "waits until" not in txt
    assert not st.needs_workspace() and st.info().n_tensors == 6 and st.info().n_launches == 2
    # a consumer over the same rows still only waits for its own workgroup, inside the launch
    soft = _p("soft_bf16", [("z", "bf16")], [("y", "softmax", ["z"], {})], [("y", "bf16")])
    c = B.dvm_encode(ctx, B.Program(soft), [B.make_shape((T, 4096))])
    st = B.dvm_stack_dependent([a, c], [-1, -1, -1, 2, -1], order_by="launch")
    assert "waits for this workgroup's own stores" in st.disasm() and st.info().n_launches == 1
