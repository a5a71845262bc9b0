"""Thin ctypes binding over libdvm.so (see include/dvm.h).  Argument marshalling only: every step
of the path (decomposition, fusion, tile planning, encoding, execution) runs in the library.

PyTorch is used by callers for device memory and streams; this module only reads
``tensor.data_ptr()``, ``tensor.shape``, ``tensor.stride()`` and the current stream handle.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdvm.so")

DVM_MAX_RANK = 6
DVM_F32, DVM_BF16 = 0, 1
DTYPES = {"f32": DVM_F32, "bf16": DVM_BF16}

# opcode values of include/dvm.h
OPCODES: Dict[str, int] = {}
for _i, _n in enumerate(["copy", "sqrt", "abs", "log", "exp", "round", "floor", "isfinite", "neg", "rsqrt", "rcp",
                         "tanh", "erf", "sigmoid", "square", "gelu_tanh", "gelu_erf", "silu", "cast"], start=1):
    OPCODES[_n] = _i
OPCODES.update({"adds": 32, "muls": 33})
for _i, _n in enumerate(["add", "sub", "mul", "div", "min", "max", "pow", "cmp_eq", "cmp_ne", "cmp_lt", "cmp_le",
                         "cmp_gt", "cmp_ge"], start=40):
    OPCODES[_n] = _i
OPCODES["select"] = 60
for _i, _n in enumerate(["sum", "rmax", "rmin", "mean", "meansq"], start=64):
    OPCODES[_n] = _i
for _i, _n in enumerate(["csum", "cmax", "cmin"], start=72):      # reductions along the penultimate axis
    OPCODES[_n] = _i
for _i, _n in enumerate(["softmax", "rmsnorm", "layernorm"], start=80):
    OPCODES[_n] = _i


class dvm_shape(C.Structure):
    _fields_ = [("rank", C.c_int32), ("align_bytes", C.c_int32),
                ("dim", C.c_int64 * DVM_MAX_RANK), ("stride", C.c_int64 * DVM_MAX_RANK)]


class dvm_code_info(C.Structure):
    _fields_ = [("kernel_type", C.c_int32), ("n_segments", C.c_int32), ("n_tensors", C.c_int32),
                ("grid", C.c_int32), ("block", C.c_int32), ("variant_k", C.c_int32), ("variant_nr", C.c_int32),
                ("n_instructions", C.c_int32), ("n_tiles", C.c_int64), ("code_bytes", C.c_int64),
                ("n_launches", C.c_int32), ("reserved", C.c_int32)]


class DvmError(RuntimeError):
    def __init__(self, status: int, where: str):
        lib = load()
        msg = lib.dvm_strerror(status).decode()
        detail = lib.dvm_last_error_detail().decode()
        super().__init__(f"{where}: {msg} ({status})" + (f": {detail}" if detail else ""))
        self.status = status


_lib = None


def load() -> C.CDLL:
    """Load libdvm.so from the package directory.  There is no fallback: without the built
    library nothing in this package can run."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2603_24239_amd.build`")
    lib = C.CDLL(_LIB_PATH)
    vp, i, sz = C.c_void_p, C.c_int, C.c_size_t
    P = C.POINTER
    sig = {
        "dvm_shape_contiguous": (i, [P(dvm_shape), i, P(C.c_int64)]),
        "dvm_ctx_create": (i, [i, P(vp)]),
        "dvm_ctx_destroy": (None, [vp]),
        "dvm_ctx_set_planner": (i, [vp, i, i]),
        "dvm_ctx_set_limits": (i, [vp, i, i]),
        "dvm_ctx_set_plan_override": (i, [vp, i, i, i]),
        "dvm_ctx_set_assignment": (i, [vp, i]),
        "dvm_ctx_set_lds_operands": (i, [vp, i]),
        "dvm_ctx_set_workspace_limit": (i, [vp, C.c_int64]),
        "dvm_ctx_set_copies_in_flight": (i, [vp, i]),
        "dvm_prog_create": (i, [P(vp)]),
        "dvm_prog_input": (i, [vp, i, P(i)]),
        "dvm_prog_op": (i, [vp, i, P(i), i, P(C.c_double), i, P(i)]),
        "dvm_prog_output": (i, [vp, i, i]),
        "dvm_prog_finish": (i, [vp]),
        "dvm_prog_num_inputs": (i, [vp]),
        "dvm_prog_num_outputs": (i, [vp]),
        "dvm_prog_destroy": (None, [vp]),
        "dvm_encode": (i, [vp, vp, P(dvm_shape), i, P(dvm_shape), vp, sz, P(sz), P(dvm_shape)]),
        "dvm_stack": (i, [P(vp), P(sz), i, vp, sz, P(sz)]),
        "dvm_stack_spatial": (i, [P(vp), P(sz), i, vp, sz, P(sz)]),
        "dvm_stack_dependent": (i, [P(vp), P(sz), i, P(i), i, i, vp, sz, P(sz)]),
        "dvm_ctx_set_sync_limit": (i, [vp, C.c_int64]),
        "dvm_workspace_status": (i, [vp, vp, P(i)]),
        "dvm_validate": (i, [vp, sz]),
        "dvm_disasm": (i, [vp, sz, C.c_char_p, sz]),
        "dvm_code_info_get": (i, [vp, sz, P(dvm_code_info)]),
        "dvm_code_tensor": (i, [vp, sz, i, P(C.c_int64), P(i), P(i), P(i)]),
        "dvm_plan": (i, [C.c_int64, i, C.c_int64, i, i, P(C.c_int64), P(C.c_int64), P(C.c_int64)]),
        "dvm_run": (i, [vp, vp, sz, P(vp), i, vp]),
        "dvm_run_static": (i, [vp, vp, sz, P(vp), i, vp]),
        "dvm_run_batched": (i, [vp, vp, sz, P(vp), i, i, vp, sz, vp]),
        "dvm_encode_timed": (i, [vp, vp, P(dvm_shape), i, P(dvm_shape), vp, sz, P(sz), i, P(C.c_int64)]),
        "dvm_copy_kernel": (i, [vp, vp, vp, sz, i, vp]),
        "dvm_strerror": (C.c_char_p, [i]),
        "dvm_last_error_detail": (C.c_char_p, []),
        "dvm_last_hip_error": (i, []),
        "dvm_fuser_create": (i, [vp, vp, P(vp)]),
        "dvm_fuser_destroy": (None, [vp]),
        "dvm_fuser_set_workspace": (i, [vp, vp, sz]),
        "dvm_fuser_tensor": (i, [vp, vp, i, P(dvm_shape), P(i)]),
        "dvm_fuser_op": (i, [vp, i, P(i), i, P(C.c_double), i, i, vp, P(i)]),
        "dvm_fuser_release": (i, [vp, i]),
        "dvm_fuser_flush": (i, [vp]),
        "dvm_fuser_stats": (i, [vp, P(C.c_int64), P(C.c_int64), P(C.c_int64), P(C.c_int64)]),
        "dvm_fuser_last_code": (i, [vp, vp, sz, P(sz)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


EXPORTED = ["dvm_shape_contiguous", "dvm_ctx_create", "dvm_ctx_destroy", "dvm_ctx_set_planner", "dvm_ctx_set_limits",
            "dvm_ctx_set_plan_override", "dvm_ctx_set_assignment", "dvm_ctx_set_lds_operands", "dvm_ctx_set_workspace_limit", "dvm_ctx_set_copies_in_flight", "dvm_prog_create",
            "dvm_prog_input", "dvm_prog_op", "dvm_prog_output", "dvm_prog_finish", "dvm_prog_num_inputs",
            "dvm_prog_num_outputs", "dvm_prog_destroy", "dvm_encode", "dvm_stack", "dvm_stack_spatial", "dvm_stack_dependent",
            "dvm_ctx_set_sync_limit", "dvm_workspace_status", "dvm_validate", "dvm_disasm",
            "dvm_code_info_get", "dvm_code_tensor", "dvm_plan", "dvm_run", "dvm_run_static", "dvm_run_batched", "dvm_encode_timed", "dvm_copy_kernel", "dvm_strerror", "dvm_last_error_detail",
            "dvm_last_hip_error", "dvm_fuser_create", "dvm_fuser_destroy", "dvm_fuser_set_workspace", "dvm_fuser_tensor", "dvm_fuser_op",
            "dvm_fuser_release", "dvm_fuser_flush", "dvm_fuser_stats", "dvm_fuser_last_code"]


def _check(status: int, where: str) -> None:
    if status != 0:
        raise DvmError(status, where)


def make_shape(dims: Sequence[int], strides: Optional[Sequence[int]] = None, align_bytes: int = 0) -> dvm_shape:
    s = dvm_shape()
    r = len(dims)
    if r > DVM_MAX_RANK:
        raise DvmError(-3, "make_shape")
    s.rank = r
    s.align_bytes = align_bytes
    if strides is None:
        arr = (C.c_int64 * max(r, 1))(*dims)
        _check(load().dvm_shape_contiguous(C.byref(s), r, arr), "dvm_shape_contiguous")
        s.align_bytes = align_bytes
    else:
        for k in range(r):
            s.dim[k] = int(dims[k])
            s.stride[k] = int(strides[k])
    return s


def _ptr_align(ptr: int) -> int:
    a = 1
    while a < 16 and ptr % (a * 2) == 0:
        a *= 2
    return a


def shape_of_tensor(t) -> dvm_shape:
    return make_shape(tuple(t.shape), tuple(t.stride()), _ptr_align(t.data_ptr()))


class Context:
    """dvm_ctx: device properties for the planner.  device=-1 builds an encode-only context."""

    def __init__(self, device: int = -1):
        self._h = C.c_void_p()
        _check(load().dvm_ctx_create(device, C.byref(self._h)), "dvm_ctx_create")
        self.device = device

    def set_planner(self, n_compute_units: int = 0, tile_overhead_elems: int = 0) -> None:
        _check(load().dvm_ctx_set_planner(self._h, n_compute_units, tile_overhead_elems), "dvm_ctx_set_planner")

    def set_limits(self, max_elems_per_lane: int = 0, max_tile_regs: int = 0) -> None:
        _check(load().dvm_ctx_set_limits(self._h, max_elems_per_lane, max_tile_regs), "dvm_ctx_set_limits")

    def set_plan_override(self, elems_per_lane: int = 0, rows_per_tile: int = 0, grid_multiplier: int = 0) -> None:
        _check(load().dvm_ctx_set_plan_override(self._h, elems_per_lane, rows_per_tile, grid_multiplier),
               "dvm_ctx_set_plan_override")

    def set_sync_limit(self, polls: int) -> None:
        _check(load().dvm_ctx_set_sync_limit(self._h, polls), "dvm_ctx_set_sync_limit")

    def set_copies_in_flight(self, copies: int) -> None:
        _check(load().dvm_ctx_set_copies_in_flight(self._h, copies), "dvm_ctx_set_copies_in_flight")

    def set_workspace_limit(self, nbytes: int) -> None:
        _check(load().dvm_ctx_set_workspace_limit(self._h, nbytes), "dvm_ctx_set_workspace_limit")

    def set_lds_operands(self, enabled) -> None:
        _check(load().dvm_ctx_set_lds_operands(self._h, int(enabled)), "dvm_ctx_set_lds_operands")

    def set_assignment(self, assignment: str) -> None:
        _check(load().dvm_ctx_set_assignment(self._h, {"blocked": 0, "interleaved": 1, "auto": 2}[assignment]), "dvm_ctx_set_assignment")

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.dvm_ctx_destroy(self._h)
            self._h = None


def _opcode(name: str, attrs) -> int:
    return OPCODES["cmp_" + str(attrs["cmp"])] if name == "cmp" else OPCODES[name]


def _immediates(name: str, attrs) -> List[float]:
    if name in ("adds", "muls"):
        return [float(attrs["imm"])]
    if name in ("rmsnorm", "layernorm"):
        return [float(attrs["eps"])]
    if name == "cast":
        return [float(DTYPES[str(attrs["to"])])]
    return []


class Program:
    """dvm_prog built from a neutral program description (workloads.programs.Program)."""

    def __init__(self, desc):
        lib = load()
        self.desc = desc
        self._h = C.c_void_p()
        _check(lib.dvm_prog_create(C.byref(self._h)), "dvm_prog_create")
        ids: Dict[str, int] = {}
        vid = C.c_int()
        for name, dt in desc.inputs:
            _check(lib.dvm_prog_input(self._h, DTYPES[dt], C.byref(vid)), "dvm_prog_input")
            ids[name] = vid.value
        for op in desc.ops:
            imm = _immediates(op.name, op.attrs)
            args = (C.c_int * max(len(op.args), 1))(*[ids[a] for a in op.args])
            immarr = (C.c_double * max(len(imm), 1))(*imm)
            _check(lib.dvm_prog_op(self._h, _opcode(op.name, op.attrs), args, len(op.args), immarr, len(imm), C.byref(vid)),
                   f"dvm_prog_op({op.name})")
            ids[op.out] = vid.value
        for name, dt in desc.outputs:
            _check(lib.dvm_prog_output(self._h, ids[name], DTYPES[dt]), "dvm_prog_output")
        _check(lib.dvm_prog_finish(self._h), "dvm_prog_finish")
        self.n_in = lib.dvm_prog_num_inputs(self._h)
        self.n_out = lib.dvm_prog_num_outputs(self._h)

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.dvm_prog_destroy(self._h)
            self._h = None


class Bytecode:
    def __init__(self, raw: bytes, out_shapes: List[Tuple[int, ...]]):
        self.raw = raw
        self._buf = C.create_string_buffer(raw, len(raw))
        self.out_shapes = out_shapes

    def __len__(self):
        return len(self.raw)

    @property
    def ptr(self):
        return C.cast(self._buf, C.c_void_p)

    def info(self) -> dvm_code_info:
        inf = dvm_code_info()
        _check(load().dvm_code_info_get(self.ptr, len(self.raw), C.byref(inf)), "dvm_code_info_get")
        return inf

    def tensor(self, index: int) -> Tuple[int, bool, int, int]:
        mb, io, dt, al = C.c_int64(), C.c_int(), C.c_int(), C.c_int()
        _check(load().dvm_code_tensor(self.ptr, len(self.raw), index, C.byref(mb), C.byref(io), C.byref(dt),
                                      C.byref(al)), "dvm_code_tensor")
        return mb.value, bool(io.value), dt.value, al.value

    def needs_workspace(self) -> bool:
        """True if the launch's last tensor is its workspace (a dependent stack with a grid-wide synchronisation point)."""
        n = self.info().n_tensors
        if n == 0:
            return False
        io = C.c_int()
        _check(load().dvm_code_tensor(self.ptr, len(self.raw), n - 1, None, C.byref(io), None, None), "dvm_code_tensor")
        return io.value == 2

    def disasm(self) -> str:
        buf = C.create_string_buffer(1 << 16)
        _check(load().dvm_disasm(self.ptr, len(self.raw), buf, len(buf)), "dvm_disasm")
        return buf.value.decode()

    def validate(self) -> None:
        _check(load().dvm_validate(self.ptr, len(self.raw)), "dvm_validate")


_ENC_CAP = 8192


def dvm_encode(ctx: Context, prog: Program, in_shapes: Sequence[dvm_shape],
               out_layout: Optional[Sequence[dvm_shape]] = None) -> Bytecode:
    lib = load()
    n = len(in_shapes)
    arr = (dvm_shape * max(n, 1))(*in_shapes)
    outl = None
    if out_layout is not None:
        outl = (dvm_shape * max(len(out_layout), 1))(*out_layout)
    buf = C.create_string_buffer(_ENC_CAP)
    ln = C.c_size_t()
    outs = (dvm_shape * max(prog.n_out, 1))()
    _check(lib.dvm_encode(ctx._h, prog._h, arr, n, outl, buf, _ENC_CAP, C.byref(ln), outs), "dvm_encode")
    shapes = [tuple(outs[i].dim[k] for k in range(outs[i].rank)) for i in range(prog.n_out)]
    return Bytecode(buf.raw[: ln.value], shapes)


def dvm_stack(codes: Sequence[Bytecode], spatial: bool = False) -> Bytecode:
    lib = load()
    n = len(codes)
    ptrs = (C.c_void_p * n)(*[c.ptr for c in codes])
    lens = (C.c_size_t * n)(*[len(c) for c in codes])
    buf = C.create_string_buffer(_ENC_CAP)
    ln = C.c_size_t()
    fn = lib.dvm_stack_spatial if spatial else lib.dvm_stack
    _check(fn(ptrs, lens, n, buf, _ENC_CAP, C.byref(ln)), "dvm_stack_spatial" if spatial else "dvm_stack")
    shapes: List[Tuple[int, ...]] = []
    for c in codes:
        shapes.extend(c.out_shapes)
    return Bytecode(buf.raw[: ln.value], shapes)


def dvm_stack_spatial(codes: Sequence[Bytecode]) -> Bytecode:
    return dvm_stack(codes, spatial=True)


def dvm_stack_dependent(codes: Sequence[Bytecode], same_as: Sequence[int], order_by: str = "kernel") -> Bytecode:
    """same_as: one entry per tensor of the launch (part after part), -1 or the index of an earlier entry that is
    the same buffer.  If the result lists a workspace (its last tensor), pass WORKSPACE_BYTES of device memory for it."""
    lib = load()
    n = len(codes)
    ptrs = (C.c_void_p * n)(*[c.ptr for c in codes])
    lens = (C.c_size_t * n)(*[len(c) for c in codes])
    sa = (C.c_int * max(len(same_as), 1))(*same_as)
    buf = C.create_string_buffer(_ENC_CAP)
    ln = C.c_size_t()
    _check(lib.dvm_stack_dependent(ptrs, lens, n, sa, len(same_as), {"kernel": 0, "launch": 1}[order_by], buf, _ENC_CAP, C.byref(ln)),
           "dvm_stack_dependent")
    shapes: List[Tuple[int, ...]] = []
    for c in codes:
        shapes.extend(c.out_shapes)
    return Bytecode(buf.raw[: ln.value], shapes)


WORKSPACE_BYTES = 256


def workspace_gave_up(workspace_ptr: int, stream: int = 0) -> bool:
    """Waits for the stream; True if a launch abandoned a synchronisation point since the workspace was cleared."""
    g = C.c_int()
    _check(load().dvm_workspace_status(C.c_void_p(workspace_ptr), C.c_void_p(stream), C.byref(g)), "dvm_workspace_status")
    return bool(g.value)


def dvm_run(ctx: Context, code: Bytecode, tensor_ptrs: Sequence[int], stream: int = 0) -> None:
    n = len(tensor_ptrs)
    arr = (C.c_void_p * max(n, 1))(*tensor_ptrs)
    _check(load().dvm_run(ctx._h, code.ptr, len(code), arr, n, C.c_void_p(stream)), "dvm_run")


def dvm_run_batched(ctx: Context, code: Bytecode, tensor_ptr_sets: Sequence[Sequence[int]], table_ptr: int, table_bytes: int,
                    stream: int = 0) -> None:
    """One launch over several sets of tensors (device pointers); `table_ptr`: device memory for the address table."""
    n_sets = len(tensor_ptr_sets)
    n = len(tensor_ptr_sets[0])
    flat = [p for s_ in tensor_ptr_sets for p in s_]
    assert len(flat) == n * n_sets
    arr = (C.c_void_p * len(flat))(*flat)
    _check(load().dvm_run_batched(ctx._h, code.ptr, len(code), arr, n, n_sets, C.c_void_p(table_ptr), table_bytes, C.c_void_p(stream)),
           "dvm_run_batched")


def dvm_run_static(ctx: Context, code: Bytecode, tensor_ptrs: Sequence[int], stream: int = 0) -> None:
    """dvm_run without the workspace entry: the library's own device array takes its place (no allocation)."""
    n = len(tensor_ptrs)
    arr = (C.c_void_p * max(n, 1))(*tensor_ptrs)
    _check(load().dvm_run_static(ctx._h, code.ptr, len(code), arr, n, C.c_void_p(stream)), "dvm_run_static")


class Fuser:
    """dvm_fuser: lazy operator buffer that fuses on arrival (argument marshalling only)."""

    _DT = {"f32": 0, "bf16": 1}

    def __init__(self, ctx: Context, stream: int = 0):
        self._h = C.c_void_p()
        self._ctx = ctx
        _check(load().dvm_fuser_create(ctx._h, C.c_void_p(stream), C.byref(self._h)), "dvm_fuser_create")

    def set_workspace(self, ptr: int, nbytes: int) -> None:
        _check(load().dvm_fuser_set_workspace(self._h, C.c_void_p(ptr), nbytes), "dvm_fuser_set_workspace")

    def tensor(self, ptr: int, dtype: str, shape: dvm_shape) -> int:
        v = C.c_int()
        _check(load().dvm_fuser_tensor(self._h, C.c_void_p(ptr), self._DT[dtype], C.byref(shape), C.byref(v)), "dvm_fuser_tensor")
        return v.value

    def op(self, name: str, args: Sequence[int], out_dtype: str, out_ptr: int, **attrs) -> int:
        imm = _immediates(name, attrs)
        arr = (C.c_int * len(args))(*args)
        immarr = (C.c_double * max(len(imm), 1))(*imm)
        v = C.c_int()
        _check(load().dvm_fuser_op(self._h, _opcode(name, attrs), arr, len(args), immarr, len(imm), self._DT[out_dtype],
                                   C.c_void_p(out_ptr), C.byref(v)), "dvm_fuser_op")
        return v.value

    def release(self, value: int) -> None:
        _check(load().dvm_fuser_release(self._h, value), "dvm_fuser_release")

    def flush(self) -> None:
        _check(load().dvm_fuser_flush(self._h), "dvm_fuser_flush")

    def stats(self) -> Dict[str, int]:
        a, b, c, d = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
        _check(load().dvm_fuser_stats(self._h, C.byref(a), C.byref(b), C.byref(c), C.byref(d)), "dvm_fuser_stats")
        return {"ops": a.value, "launches": b.value, "flushes": c.value, "elided": d.value}

    def last_code(self) -> "Bytecode":
        buf = C.create_string_buffer(_ENC_CAP)
        ln = C.c_size_t()
        _check(load().dvm_fuser_last_code(self._h, buf, _ENC_CAP, C.byref(ln)), "dvm_fuser_last_code")
        return Bytecode(buf.raw[: ln.value], [])

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.dvm_fuser_destroy(self._h)
            self._h = None


def dvm_plan(total: int, n_cores: int, t_max: int, align: int, overhead: int = 2) -> Tuple[int, int, int]:
    a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
    _check(load().dvm_plan(total, n_cores, t_max, align, overhead, C.byref(a), C.byref(b), C.byref(c)), "dvm_plan")
    return a.value, b.value, c.value


# ------------------------------------------------------------------------------------------------
# convenience for torch callers: marshal tensors, allocate outputs (torch owns device memory)
# ------------------------------------------------------------------------------------------------

def encode_for(ctx: Context, prog: Program, inputs: Sequence, outputs: Optional[Sequence] = None) -> Bytecode:
    """Encode `prog` for the shapes/strides of the given torch tensors (and output views, if any)."""
    in_shapes = [shape_of_tensor(t) for t in inputs]
    out_layout = [shape_of_tensor(t) for t in outputs] if outputs is not None else None
    return dvm_encode(ctx, prog, in_shapes, out_layout)


def check_buffers(code: Bytecode, tensors: Sequence) -> None:
    """Host-side guard: every tensor's storage must cover what the bytecode will touch."""
    for i, t in enumerate(tensors):
        need, _is_out, _dt, _al = code.tensor(i)
        have = (t.untyped_storage().nbytes() - t.storage_offset() * t.element_size()) if t.numel() else 0
        if need > have:
            raise DvmError(-1, f"tensor {i}: bytecode touches {need} bytes, storage holds {have}")


def run_on(ctx: Context, code: Bytecode, tensors: Sequence, stream: Optional[int] = None) -> None:
    import torch
    check_buffers(code, tensors)
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    dvm_run(ctx, code, [t.data_ptr() for t in tensors], stream)
