"""Operator programs as plain data.

A program is a list of named inputs (with storage dtype), a list of ops in SSA form and a list of
named outputs (with storage dtype).  Op names follow the paper's Table 1 (tile-level virtual
instructions) in lower case, plus a few compound ops that the front end decomposes into basic ops
(Section 3, "decomposed into basic operators").

Vocabulary (all elementwise ops broadcast NumPy-style; reductions act on the last axis and keep it
with extent 1, i.e. Table 1's Sum/Max/Min on [M, size, 1]):

  unary      copy sqrt abs log exp round floor isfinite neg rsqrt rcp tanh erf sigmoid square
             gelu_tanh gelu_erf silu cast(to=)
  scalar     adds(imm=) muls(imm=)
  binary     add sub mul div min max pow cmp(cmp=eq|ne|lt|le|gt|ge)
  ternary    select(cond, a, b)
  reduce     sum rmax rmin mean meansq
  compound   softmax  rmsnorm(x, w; eps=)  layernorm(x, gamma, beta; eps=)
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple


@dataclass(frozen=True)
class Op:
    out: str
    name: str
    args: Tuple[str, ...]
    attrs: Dict[str, object] = field(default_factory=dict)


@dataclass(frozen=True)
class Program:
    name: str
    inputs: Tuple[Tuple[str, str], ...]      # (value name, storage dtype "f32" | "bf16")
    ops: Tuple[Op, ...]
    outputs: Tuple[Tuple[str, str], ...]     # (value name, storage dtype)


def _p(name, inputs, ops, outputs) -> Program:
    return Program(name, tuple(inputs), tuple(Op(o, n, tuple(a), dict(k)) for (o, n, a, k) in ops),
                   tuple(outputs))


def _build() -> Dict[str, Program]:
    P: Dict[str, Program] = {}

    # config 1: y = gelu(x*a + b), fp32; erf form (the unqualified textbook GELU), tanh form as a variant
    for variant in ("erf", "tanh"):
        P[f"c1_gelu_{variant}"] = _p(
            f"c1_gelu_{variant}", [("x", "f32"), ("a", "f32"), ("b", "f32")],
            [("t", "mul", ["x", "a"], {}), ("u", "add", ["t", "b"], {}), ("y", f"gelu_{variant}", ["u"], {})],
            [("y", "f32")])

    # config 2: RMSNorm with learned scale, bf16 storage, eps 1e-6 -- compound form and spelled-out form
    P["c2_rmsnorm"] = _p("c2_rmsnorm", [("x", "bf16"), ("w", "bf16")],
                         [("y", "rmsnorm", ["x", "w"], {"eps": 1e-6})], [("y", "bf16")])
    P["c2_rmsnorm_basic"] = _p(
        "c2_rmsnorm_basic", [("x", "bf16"), ("w", "bf16")],
        [("ms", "meansq", ["x"], {}), ("v", "adds", ["ms"], {"imm": 1e-6}), ("r", "rsqrt", ["v"], {}),
         ("n", "mul", ["x", "r"], {}), ("y", "mul", ["n", "w"], {})],
        [("y", "bf16")])

    # config 3: masked softmax fp32: add -> rowmax -> sub -> exp -> rowsum -> div
    P["c3_masked_softmax"] = _p(
        "c3_masked_softmax", [("z", "f32"), ("mask", "f32")],
        [("s", "add", ["z", "mask"], {}), ("m", "rmax", ["s"], {}), ("d", "sub", ["s", "m"], {}),
         ("e", "exp", ["d"], {}), ("l", "sum", ["e"], {}), ("p", "div", ["e", "l"], {})],
        [("p", "f32")])
    P["softmax_f32"] = _p("softmax_f32", [("z", "f32")], [("p", "softmax", ["z"], {})], [("p", "f32")])
    P["softmax_bf16"] = _p("softmax_bf16", [("z", "bf16")], [("p", "softmax", ["z"], {})], [("p", "bf16")])

    # config 4: the 12-op transformer non-GEMM chain, bf16 storage, LayerNorm eps 1e-5
    P["c4_chain"] = _p(
        "c4_chain",
        [("x", "bf16"), ("r", "bf16"), ("gamma", "bf16"), ("beta", "bf16"), ("bias", "bf16"), ("mask", "bf16")],
        [("h", "add", ["x", "r"], {}),              # 1 residual add
         ("mu", "mean", ["h"], {}),                 # 2
         ("d", "sub", ["h", "mu"], {}),             # 3
         ("v", "meansq", ["d"], {}),                # 4
         ("ve", "adds", ["v"], {"imm": 1e-5}),
         ("s", "rsqrt", ["ve"], {}),                # 5 (rsqrt(v+eps))
         ("n", "mul", ["d", "s"], {}),              # 6
         ("ng", "mul", ["n", "gamma"], {}),         # 7
         ("nb", "add", ["ng", "beta"], {}),         # 8
         ("nc", "add", ["nb", "bias"], {}),         # 9 bias add
         ("g", "gelu_tanh", ["nc"], {}),            # 10
         ("gm", "mul", ["g", "mask"], {}),          # 11 dropout mask
         ("y", "add", ["gm", "h"], {})],            # 12 final residual add
        [("y", "bf16")])
    # the same chain with the compound LayerNorm op
    P["c4_chain_ln"] = _p(
        "c4_chain_ln",
        [("x", "bf16"), ("r", "bf16"), ("gamma", "bf16"), ("beta", "bf16"), ("bias", "bf16"), ("mask", "bf16")],
        [("h", "add", ["x", "r"], {}), ("nb", "layernorm", ["h", "gamma", "beta"], {"eps": 1e-5}),
         ("nc", "add", ["nb", "bias"], {}), ("g", "gelu_tanh", ["nc"], {}), ("gm", "mul", ["g", "mask"], {}),
         ("y", "add", ["gm", "h"], {})],
        [("y", "bf16")])

    # config 5: the six per-layer programs
    P["c5_rmsnorm"] = _p("c5_rmsnorm", [("x", "bf16"), ("w", "bf16")],
                         [("y", "rmsnorm", ["x", "w"], {"eps": 1e-6})], [("y", "bf16")])
    # RoPE, rotate-half pairing; x1/x2 are the two halves of the head dim passed as strided views,
    # cos/sin are fp32 tables broadcast over heads; y1/y2 are written into the halves of the output
    P["c5_rope"] = _p(
        "c5_rope", [("x1", "bf16"), ("x2", "bf16"), ("cos", "f32"), ("sin", "f32")],
        [("a", "mul", ["x1", "cos"], {}), ("b", "mul", ["x2", "sin"], {}), ("y1", "sub", ["a", "b"], {}),
         ("c", "mul", ["x2", "cos"], {}), ("d", "mul", ["x1", "sin"], {}), ("y2", "add", ["c", "d"], {})],
        [("y1", "bf16"), ("y2", "bf16")])
    P["c5_softmax"] = P["softmax_bf16"]
    P["c5_residual"] = _p("c5_residual", [("a", "bf16"), ("b", "bf16")], [("y", "add", ["a", "b"], {})],
                          [("y", "bf16")])
    P["c5_silu_gate"] = _p("c5_silu_gate", [("g", "bf16"), ("u", "bf16")],
                           [("s", "silu", ["g"], {}), ("y", "mul", ["s", "u"], {})], [("y", "bf16")])

    # the paper's own subgraph workloads (Table 2): LayerNorm and if-else-add  (a > b ? 2x : 4x) + y
    P["layernorm_f32"] = _p("layernorm_f32", [("x", "f32"), ("gamma", "f32"), ("beta", "f32")],
                            [("y", "layernorm", ["x", "gamma", "beta"], {"eps": 1e-5})], [("y", "f32")])
    P["layernorm_bf16"] = _p("layernorm_bf16", [("x", "bf16"), ("gamma", "bf16"), ("beta", "bf16")],
                             [("y", "layernorm", ["x", "gamma", "beta"], {"eps": 1e-5})], [("y", "bf16")])
    P["if_else_add"] = _p(
        "if_else_add", [("a", "f32"), ("b", "f32"), ("x", "f32"), ("y", "f32")],
        [("c", "cmp", ["a", "b"], {"cmp": "gt"}), ("x2", "muls", ["x"], {"imm": 2.0}),
         ("x4", "muls", ["x"], {"imm": 4.0}), ("s", "select", ["c", "x2", "x4"], {}),
         ("o", "add", ["s", "y"], {})],
        [("o", "f32")])
    # the two resolved branches of if-else-add (control flow decided on the host, Section 6)
    for nm, k in (("true", 2.0), ("false", 4.0)):
        P[f"if_else_add_{nm}"] = _p(f"if_else_add_{nm}", [("x", "f32"), ("y", "f32")],
                                    [("t", "muls", ["x"], {"imm": k}), ("o", "add", ["t", "y"], {})],
                                    [("o", "f32")])

    # reductions along the penultimate axis (Table 1's Sum / Max / Min over [M, size, N]): a plain column sum,
    # a bias gradient (bf16 in, fp32 out), a full-size output beside the reduction, and an epilogue of ops on
    # the reduced values
    P["colsum"] = _p("colsum", [("x", "f32")], [("s", "csum", ["x"], {})], [("s", "f32")])
    P["bias_grad_bf16"] = _p("bias_grad_bf16", [("dy", "bf16")], [("db", "csum", ["dy"], {})], [("db", "f32")])
    P["colsum_exp"] = _p("colsum_exp", [("x", "f32")],
                         [("e", "exp", ["x"], {}), ("s", "csum", ["e"], {})], [("e", "f32"), ("s", "f32")])
    P["col_stats"] = _p(
        "col_stats", [("x", "f32"), ("b", "f32")],
        [("q", "square", ["x"], {}), ("s", "csum", ["q"], {}), ("m", "muls", ["s"], {"imm": 0.125}),
         ("r", "sqrt", ["m"], {}), ("o", "add", ["r", "b"], {}),
         ("hi", "cmax", ["x"], {}), ("lo", "cmin", ["x"], {}), ("w", "sub", ["hi", "lo"], {})],
        [("o", "f32"), ("w", "f32")])

    # small programs used by pins and unit tests
    P["identity_affine"] = _p("identity_affine", [("x", "f32")],
                              [("t", "muls", ["x"], {"imm": 1.0}), ("y", "adds", ["t"], {"imm": 0.0})],
                              [("y", "f32")])
    P["add_sqrt"] = _p("add_sqrt", [("a", "f32"), ("b", "f32")],
                       [("c", "add", ["a", "b"], {}), ("d", "sqrt", ["c"], {})], [("d", "f32")])
    P["add_f16like"] = _p("add_f16like", [("a", "bf16"), ("b", "bf16")], [("c", "add", ["a", "b"], {})],
                          [("c", "bf16")])
    return P


PROGRAMS: Dict[str, Program] = _build()


def get_program(name: str) -> Program:
    return PROGRAMS[name]


def single_op_program(op: str, n_args: int, dtype: str = "f32", **attrs) -> Program:
    """A one-op program `y = op(a0, a1, ...)`, used by per-op parity tests."""
    names: List[str] = [f"a{i}" for i in range(n_args)]
    return _p(f"single_{op}", [(n, dtype) for n in names], [("y", op, names, attrs)], [("y", dtype)])
