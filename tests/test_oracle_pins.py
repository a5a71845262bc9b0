"""Pins for the CPU oracle: values the paper prints, closed forms, invariants, brute force on tiny
inputs and independent library routines.  None of these tests touches the HIP path."""
import itertools
import math
import os
import zlib

import numpy as np
import pytest
import torch

from oracle import interp, tiling
from workloads import programs as W
from workloads.programs import single_op_program

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _kv(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, v = [s.strip() for s in line.split("=")]
        out[k] = int(v)
    return out


def run(prog, **inputs):
    rounded, exact = interp.run(prog, inputs)
    return rounded, exact


# ------------------------------------------------------------------ tile planner (Section 4.2 example)

def test_tile_planner_worked_example():
    g = _kv(os.path.join(GOLD, "tile_example.txt"))
    total = g["rows"] * g["cols"]
    align = g["instr_width_bytes"] // g["elem_bytes"]
    t, ta = tiling.hardware_align_div(total, g["n_cores"], t_max=1 << 20, align=align)
    assert t == g["min_cost_tile"]
    assert ta == g["aligned_tile"]
    tiles = tiling.tiles_of(total, t)
    assert len(tiles) == g["n_tiles"]
    assert tiles[-1][1] - tiles[-1][0] == g["tail_tile"]
    # after rounding: still 40 tiles, tail unpadded
    tiles_a = tiling.tiles_of(total, ta)
    assert len(tiles_a) == g["n_tiles"]
    assert tiles_a[-1][1] == total and tiles_a[-1][1] - tiles_a[-1][0] == total - 39 * ta
    # one wave of 40 tiles (cost 822) beats the two-wave optimum (2 * 412 = 824)
    assert tiling.tile_cost(total, 820, 40) == 822
    assert tiling.tile_cost(total, 410, 40) == 824
    # Algorithm 1 on the collapsed (one-dimensional) space gives the same aligned tile
    assert tiling.shape_tiling([total], 1 << 20, g["n_cores"], align) == [ta]


def test_tile_cost_model_properties():
    rng = np.random.default_rng(1)
    for _ in range(200):
        total = int(rng.integers(1, 5000))
        n = int(rng.integers(1, 64))
        tmax = int(rng.integers(1, 3000))
        align = int(rng.choice([1, 2, 4, 8, 16]))
        t, ta = tiling.hardware_align_div(total, n, tmax, align)
        assert 1 <= t <= min(tmax, total)
        # optimality against every candidate
        c = tiling.tile_cost(total, t, n)
        assert all(c <= tiling.tile_cost(total, u, n) for u in range(1, min(tmax, total) + 1))
        # alignment respects the limit
        assert ta <= max(tmax, t)
        if ta != t:
            assert ta % align == 0
        tl = tiling.tiles_of(total, ta)
        assert tl[0][0] == 0 and tl[-1][1] == total
        assert all(a[1] == b[0] for a, b in zip(tl, tl[1:]))
        assert all(e - s == ta for s, e in tl[:-1])


def test_alg1_outer_dims_get_extent_one():
    # inner remainder larger than T_max -> that dimension is tiled to 1; first fitting dim is split
    tile = tiling.shape_tiling([6, 50, 1000], t_max=4000, n_cores=8, align=16)
    assert tile[0] == 1 and 1 <= tile[1] <= 4 and tile[2] == 1000
    tile = tiling.shape_tiling([6, 50, 1000], t_max=500, n_cores=8, align=16)
    assert tile[0] == 1 and tile[1] == 1 and tile[2] <= 500 and tile[2] % 16 == 0


def test_alg2_assignment_partitions_tiles():
    for M in range(0, 201):
        for N in range(1, 65):
            seen = []
            for cid in range(N):
                lo, hi = tiling.vm_tile_range(M, N, cid)
                assert lo <= hi
                seen.extend(range(lo, hi))
            assert seen == list(range(M))
    assert tiling.vm_tile_range(10, 4, 0) == (0, 3)
    assert tiling.vm_tile_range(10, 4, 3) == (9, 10)


def test_interleaved_assignment_partitions_tiles_like_the_blocked_one():
    for M in list(range(0, 80)) + [199, 200]:
        for N in (1, 2, 3, 7, 40, 64):
            seen = []
            for cid in range(N):
                mine = tiling.interleaved_tiles(M, N, cid)
                lo, hi = tiling.vm_tile_range(M, N, cid)
                # as many tiles as Algorithm 2's m = ceil(M/N), or fewer; never more than one apart between cores
                assert len(mine) <= tiling.ceil_div(M, N) if M else not mine
                assert all(b - a == N for a, b in zip(mine, mine[1:]))
                seen += mine
                assert hi - lo <= tiling.ceil_div(M, N) if M else hi == lo
            assert sorted(seen) == list(range(M))
            counts = [len(tiling.interleaved_tiles(M, N, c)) for c in range(N)]
            assert max(counts) - min(counts) <= 1


# ------------------------------------------------------------------ storage rounding

def test_bf16_rounding_matches_library_and_ties_to_even():
    g = torch.Generator().manual_seed(7)
    x = torch.randn(20000, generator=g) * torch.exp(torch.randn(20000, generator=g) * 20)
    x = torch.cat([x, torch.tensor([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 3.4e38, 1e-40,
                                    9.1835e-41, float("inf"), float("-inf")])])
    want = x.to(torch.bfloat16).to(torch.float64).numpy()
    got = interp.round_to_bf16(x.to(torch.float64).numpy())
    assert np.array_equal(got, want)
    # ties: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    assert interp.round_to_bf16(1.0 + 2.0 ** -8) == 1.0
    assert interp.round_to_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert np.isnan(interp.round_to_bf16(np.nan))
    assert interp.round_to_bf16(1.0 / 0.9) == 1.109375


# ------------------------------------------------------------------ every elementwise op: brute force

_SCALAR = {
    "copy": lambda a: a, "sqrt": lambda a: math.sqrt(a) if a >= 0 else float("nan"),
    "abs": abs, "log": lambda a: math.log(a) if a > 0 else (float("-inf") if a == 0 else float("nan")),
    "exp": math.exp, "neg": lambda a: -a, "rsqrt": lambda a: 1.0 / math.sqrt(a), "rcp": lambda a: 1.0 / a,
    "tanh": math.tanh, "erf": math.erf, "sigmoid": lambda a: 1.0 / (1.0 + math.exp(-a)),
    "square": lambda a: a * a, "floor": math.floor,
    "gelu_tanh": lambda u: 0.5 * u * (1 + math.tanh(math.sqrt(2 / math.pi) * (u + 0.044715 * u * u * u))),
    "gelu_erf": lambda u: 0.5 * u * (1 + math.erf(u / math.sqrt(2))),
    "silu": lambda g: g / (1.0 + math.exp(-g)),
    "add": lambda a, b: a + b, "sub": lambda a, b: a - b, "mul": lambda a, b: a * b,
    "div": lambda a, b: a / b, "min": min, "max": max, "pow": lambda a, b: math.pow(abs(a), b),
}
_POSITIVE = {"sqrt", "log", "rsqrt"}


@pytest.mark.parametrize("op", sorted(_SCALAR))
def test_elementwise_ops_bruteforce_with_broadcast(op):
    fn = _SCALAR[op]
    nargs = fn.__code__.co_argcount if hasattr(fn, "__code__") else 1
    if op in ("abs",):
        nargs = 1
    if op in ("min", "max"):
        nargs = 2
    rng = np.random.default_rng(zlib.crc32(op.encode()) % 1000)      # (the same inputs in every process: str hashes are salted)
    shape_sets = [[(1,)], [(1, 1)], [(2, 3)], [(3, 1, 5), (1, 4, 1)]]
    for shapes in shape_sets:
        shapes = (shapes * 2)[:nargs] if len(shapes) >= nargs else (shapes * nargs)[:nargs]
        arrs = []
        for s in shapes:
            a = rng.standard_normal(s).astype(np.float32).astype(np.float64)
            if op in _POSITIVE or op == "pow":
                a = np.abs(a) + 0.25
            arrs.append(a)
        prog = single_op_program(op, nargs)
        _, exact = run(prog, **{f"a{i}": a for i, a in enumerate(arrs)})
        got = exact["y"]
        bshape = np.broadcast_shapes(*[a.shape for a in arrs])
        assert got.shape == bshape
        barrs = [np.broadcast_to(a, bshape) for a in arrs]
        for idx in itertools.product(*[range(n) for n in bshape]):
            want = fn(*[float(b[idx]) for b in barrs])
            assert got[idx] == pytest.approx(want, rel=1e-14, abs=1e-300), (op, idx)


def _c_pow(a, b):
    try:
        return math.pow(a, b)
    except ValueError:          # the C library's domain error: a finite negative base with a non-integer exponent
        return float("nan")
    except OverflowError:       # (math.pow raises where the C library returns an infinity)
        return float("inf") if not (a < 0 and float(b).is_integer() and int(b) % 2 == 1) else float("-inf")


def test_pow_min_max_special_values():
    # Pow on negative bases, zeros, infinities and NaN against the C library's pow (through math.pow)
    bases = [-8.0, -2.5, -1.0, -0.5, 0.0, 0.5, 1.0, 2.0, 9.0, math.inf, -math.inf, math.nan]
    exps = [-3.0, -2.0, -1.0, -0.5, 0.0, 0.5, 1.0, 2.0, 3.0, 4.0, 2.5, 17.0, math.inf, -math.inf, math.nan]
    a = np.array(bases)[:, None] * np.ones((1, len(exps)))
    b = np.ones((len(bases), 1)) * np.array(exps)[None, :]
    _, ex = run(single_op_program("pow", 2), a0=a, a1=b)
    for i, x in enumerate(bases):
        for j, y in enumerate(exps):
            if x == 0.0 and y < 0:
                want = math.inf          # (math.pow raises for a zero base with a negative exponent; C returns +inf for +0)
            else:
                want = _c_pow(x, y)
            got = ex["y"][i, j]
            assert (math.isnan(got) and math.isnan(want)) or got == pytest.approx(want, rel=1e-15), (x, y, got, want)
    # (-2)^3 = -8, (-2)^2 = 4, (-8)^(1/3) is not a real power: NaN
    _, ex = run(single_op_program("pow", 2), a0=np.array([-2.0, -2.0, -8.0]), a1=np.array([3.0, 2.0, 1.0 / 3.0]))
    assert ex["y"][0] == -8.0 and ex["y"][1] == 4.0 and math.isnan(ex["y"][2])
    # Min / Max propagate a NaN operand, element-wise and as reductions along either axis
    x = np.array([[1.0, math.nan, -math.inf, 0.0], [2.0, 3.0, math.inf, -0.0]])
    y = np.array([[math.nan, 5.0, 7.0, 1.0], [1.0, 4.0, 2.0, 0.0]])
    for op, pick in (("max", max), ("min", min)):
        _, ex = run(single_op_program(op, 2), a0=x, a1=y)
        for idx in itertools.product(range(2), range(4)):
            u, v = x[idx], y[idx]
            want = math.nan if (math.isnan(u) or math.isnan(v)) else pick(u, v)
            got = ex["y"][idx]
            assert (math.isnan(got) and math.isnan(want)) or got == want, (op, idx)
    for op, axis, pick in (("rmax", -1, max), ("rmin", -1, min), ("cmax", -2, max), ("cmin", -2, min)):
        _, ex = run(single_op_program(op, 1), a0=x)
        lines = x if axis == -1 else x.T
        want = [math.nan if any(math.isnan(t) for t in line) else pick(line) for line in lines]
        got = ex["y"].reshape(-1)
        assert len(got) == len(want)
        for g_, w_ in zip(got, want):
            assert (math.isnan(g_) and math.isnan(w_)) or g_ == w_, (op, got, want)


def test_row_scale_hand_computed():
    # RMS over the finite entries of each row (last axis), kept with extent 1: rows (3, 4, inf) and (nan, 0, -6)
    x = np.array([[3.0, 4.0, math.inf], [math.nan, 0.0, -6.0]])
    s = interp.row_scale(x)
    assert s.shape == (2, 1)
    assert s[0, 0] == pytest.approx(math.sqrt((9 + 16) / 2), rel=1e-15)
    assert s[1, 0] == pytest.approx(math.sqrt(36 / 2), rel=1e-15)
    # a wrong axis would give per-column values: shape (1, 3)
    x3 = np.arange(24, dtype=np.float64).reshape(2, 3, 4)
    s3 = interp.row_scale(x3)
    assert s3.shape == (2, 3, 1)
    for i in range(2):
        for j in range(3):
            assert s3[i, j, 0] == pytest.approx(math.sqrt(sum(v * v for v in x3[i, j]) / 4), rel=1e-15)
    # a row without any finite entry has scale 0
    assert interp.row_scale(np.array([[math.nan, math.inf]]))[0, 0] == 0.0


def test_ops_against_torch_cpu_float64():
    g = torch.Generator().manual_seed(3)
    x = torch.randn(7, 33, generator=g, dtype=torch.float64)
    y = torch.randn(7, 33, generator=g, dtype=torch.float64)
    F = torch.nn.functional
    table = {
        "exp": torch.exp(x), "tanh": torch.tanh(x), "erf": torch.erf(x), "sigmoid": torch.sigmoid(x),
        "gelu_erf": F.gelu(x), "gelu_tanh": F.gelu(x, approximate="tanh"), "silu": F.silu(x),
        "abs": x.abs(), "floor": x.floor(), "round": x.float().round().double(), "neg": -x,
    }
    for op, want in table.items():
        _, ex = run(single_op_program(op, 1), a0=x.numpy())
        np.testing.assert_allclose(ex["y"], want.numpy(), rtol=1e-12, atol=1e-14, err_msg=op)
    table2 = {"add": x + y, "sub": x - y, "mul": x * y, "div": x / y, "min": torch.minimum(x, y),
              "max": torch.maximum(x, y)}
    for op, want in table2.items():
        _, ex = run(single_op_program(op, 2), a0=x.numpy(), a1=y.numpy())
        np.testing.assert_allclose(ex["y"], want.numpy(), rtol=1e-14, err_msg=op)
    for c, tfn in (("eq", torch.eq), ("ne", torch.ne), ("lt", torch.lt), ("le", torch.le), ("gt", torch.gt),
                   ("ge", torch.ge)):
        yy = y.clone()
        yy[:, ::3] = x[:, ::3]
        _, ex = run(single_op_program("cmp", 2, cmp=c), a0=x.float().double().numpy(),
                    a1=yy.float().double().numpy())
        assert np.array_equal(ex["y"], tfn(x.float(), yy.float()).double().numpy()), c
    cond = (torch.rand(7, 33, generator=g) > 0.5).double()
    _, ex = run(single_op_program("select", 3), a0=cond.numpy(), a1=x.numpy(), a2=y.numpy())
    assert np.array_equal(ex["y"], torch.where(cond != 0, x, y).numpy())
    # reductions over the last axis, kept
    for op, want in (("sum", x.sum(-1, keepdim=True)), ("rmax", x.amax(-1, keepdim=True)),
                     ("rmin", x.amin(-1, keepdim=True)), ("mean", x.mean(-1, keepdim=True)),
                     ("meansq", (x * x).mean(-1, keepdim=True))):
        _, ex = run(single_op_program(op, 1), a0=x.numpy())
        assert ex["y"].shape == (7, 1)
        np.testing.assert_allclose(ex["y"], want.numpy(), rtol=1e-13, err_msg=op)
    _, ex = run(single_op_program("isfinite", 1), a0=np.array([1.0, np.inf, -np.inf, np.nan, 1e39, -3.0]))
    assert ex["y"].tolist() == [1, 0, 0, 0, 0, 1]      # 1e39 overflows fp32, the deciding precision
    _, ex = run(single_op_program("round", 1), a0=np.array([0.5, 1.5, 2.5, -0.5, -1.5, 2.4999, 2.5001]))
    assert ex["y"].tolist() == [0, 2, 2, -0.0, -2, 2, 3]
    _, ex = run(single_op_program("cast", 1, to="bf16"), a0=np.array([1.0 / 0.9, 1 + 2.0 ** -8]))
    assert ex["y"].tolist() == [1.109375, 1.0]
    _, ex = run(single_op_program("adds", 1, imm=2.5), a0=np.array([1.0, -2.5]))
    assert ex["y"].tolist() == [3.5, 0.0]
    _, ex = run(single_op_program("muls", 1, imm=-2.0), a0=np.array([1.0, -2.5]))
    assert ex["y"].tolist() == [-2.0, 5.0]


# ------------------------------------------------------------------ identity, GELU, SiLU

def test_identity_program_is_bit_exact():
    x = torch.randn(5, 17, generator=torch.Generator().manual_seed(0)).numpy()
    x[0, 0], x[0, 1] = 0.0, -0.0
    rounded, _ = run(W.get_program("identity_affine"), x=x)
    assert np.array_equal(rounded["y"].astype(np.float32).view(np.uint32)[x != 0],
                          x.view(np.uint32)[x != 0])
    assert np.all(rounded["y"][x == 0] == 0)


@pytest.mark.parametrize("variant", ["gelu_erf", "gelu_tanh"])
def test_gelu_closed_forms(variant):
    u = np.linspace(-6, 6, 241)
    _, ex = run(single_op_program(variant, 1), a0=u)
    _, exn = run(single_op_program(variant, 1), a0=-u)
    assert ex["y"][120] == 0.0                                         # gelu(0) = 0
    np.testing.assert_allclose(ex["y"] - exn["y"], u, rtol=0, atol=1e-15)   # gelu(u) - gelu(-u) = u
    big = np.array([10.0, 20.0, -10.0, -20.0])
    r, _ = run(single_op_program(variant, 1), a0=big)
    assert r["y"].tolist() == [10.0, 20.0, 0.0, 0.0] or np.allclose(r["y"], [10, 20, 0, 0], atol=1e-20)
    # the two variants differ (so the program text must say which one is meant)
    _, a = run(single_op_program("gelu_erf", 1), a0=np.array([1.0]))
    _, b = run(single_op_program("gelu_tanh", 1), a0=np.array([1.0]))
    assert 1e-5 < abs(a["y"][0] - b["y"][0]) < 1e-3
    assert a["y"][0] == pytest.approx(0.8413447460685429, rel=1e-15)    # Phi(1)


def test_silu_closed_forms():
    g = np.linspace(-8, 8, 161)
    _, ex = run(single_op_program("silu", 1), a0=g)
    _, exn = run(single_op_program("silu", 1), a0=-g)
    assert ex["y"][80] == 0.0
    np.testing.assert_allclose(ex["y"] - exn["y"], g, atol=1e-15)


def test_c1_program_matches_manual():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((4, 10)).astype(np.float32).astype(np.float64)
    a = rng.uniform(-1, 1, 10).astype(np.float32).astype(np.float64)
    b = rng.uniform(-1, 1, 10).astype(np.float32).astype(np.float64)
    _, ex = run(W.get_program("c1_gelu_erf"), x=x, a=a, b=b)
    for i in range(4):
        for j in range(10):
            u = x[i, j] * a[j] + b[j]
            assert ex["y"][i, j] == pytest.approx(0.5 * u * (1 + math.erf(u / math.sqrt(2))), rel=1e-14)


# ------------------------------------------------------------------ softmax

def test_softmax_invariants():
    rng = np.random.default_rng(5)
    z = (rng.standard_normal((3, 4, 37)) * 3).astype(np.float32).astype(np.float64)
    prog = W.get_program("softmax_f32")
    _, ex = run(prog, z=z)
    p = ex["p"]
    assert p.shape == z.shape
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-12)
    _, ex2 = run(prog, z=z + 11.5)
    np.testing.assert_allclose(ex2["p"], p, rtol=1e-12)                 # shift invariance
    _, ex3 = run(prog, z=np.full((2, 9), -3.25))
    np.testing.assert_allclose(ex3["p"], 1.0 / 9, rtol=1e-15)           # constant row
    want = torch.softmax(torch.from_numpy(z), -1).numpy()
    np.testing.assert_allclose(p, want, rtol=1e-12)
    # rows are independent: softmax acts on the LAST axis only
    _, ex4 = run(prog, z=z[1:2])
    np.testing.assert_array_equal(ex4["p"], p[1:2])


def test_masked_softmax_causal_equal_scores():
    S = 9
    z = np.zeros((2, 3, S, S))
    mask = np.triu(np.full((S, S), -np.inf), 1)
    _, ex = run(W.get_program("c3_masked_softmax"), z=z, mask=mask)
    p = ex["p"]
    for i in range(S):
        np.testing.assert_allclose(p[..., i, : i + 1], 1.0 / (i + 1), rtol=1e-15)
        assert np.all(p[..., i, i + 1:] == 0.0)                         # exactly zero above the diagonal
    assert np.all(p[..., 0, 0] == 1.0)                                  # row 0 is one-hot
    # a fully masked row is NaN (documented reading of -inf arithmetic)
    _, exn = run(W.get_program("c3_masked_softmax"), z=np.zeros((1, 1, 2, 2)), mask=np.full((2, 2), -np.inf))
    assert np.all(np.isnan(exn["p"]))
    # spelled-out 6-op program == compound softmax on z + mask
    rng = np.random.default_rng(2)
    zz = rng.standard_normal((2, 2, S, S)) * 3
    _, e1 = run(W.get_program("c3_masked_softmax"), z=zz, mask=mask)
    _, e2 = run(W.get_program("softmax_f32"), z=zz + mask)
    np.testing.assert_allclose(e1["p"], e2["p"], rtol=1e-14)


# ------------------------------------------------------------------ RMSNorm / LayerNorm

def _rms(a):
    return np.sqrt((a * a).mean(-1, keepdims=True))


def test_rmsnorm_invariants():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((3, 5, 64))
    ones = np.ones(64)
    import dataclasses
    base = W.get_program("c2_rmsnorm")
    p0 = dataclasses.replace(base, ops=(W.Op("y", "rmsnorm", ("x", "w"), {"eps": 0.0}),))
    _, ex = run(p0, x=x, w=ones)
    np.testing.assert_allclose(_rms(ex["y"]), 1.0, rtol=1e-13)           # unit RMS for w=1, eps=0
    _, ex2 = run(p0, x=7.5 * x, w=ones)
    np.testing.assert_allclose(ex2["y"], ex["y"], rtol=1e-13)            # scale invariance
    w = rng.standard_normal(64)
    _, ex3 = run(p0, x=np.full((2, 64), -2.0), w=w)
    np.testing.assert_allclose(ex3["y"], -np.broadcast_to(w, (2, 64)), rtol=1e-14)  # constant row -> sign(c) w
    eps = 1e-6
    _, ex4 = run(base, x=x, w=w)
    ms = (x * x).mean(-1, keepdims=True)
    np.testing.assert_allclose(_rms(ex4["y"] / w), np.sqrt(ms / (ms + eps)), rtol=1e-13)
    # compound op == spelled-out basic ops
    _, ex5 = run(W.get_program("c2_rmsnorm_basic"), x=x, w=w)
    np.testing.assert_allclose(ex5["y"], ex4["y"], rtol=1e-14)
    # against the library (torch >= 2.4 has rms_norm)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(w), eps=eps).numpy()
    np.testing.assert_allclose(ex4["y"], want, rtol=1e-12)


def test_layernorm_invariants():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((4, 6, 48)) * 2 + 0.7
    prog = W.get_program("layernorm_f32")
    eps = 1e-5
    _, ex = run(prog, x=x, gamma=np.ones(48), beta=np.zeros(48))
    y = ex["y"]
    np.testing.assert_allclose(y.mean(-1), 0.0, atol=1e-14)
    v = x.var(-1, keepdims=True)                                        # biased variance
    np.testing.assert_allclose(y.var(-1, keepdims=True), v / (v + eps), rtol=1e-12)
    _, ex2 = run(prog, x=x + 123.0, gamma=np.ones(48), beta=np.zeros(48))
    np.testing.assert_allclose(ex2["y"], y, atol=1e-10)                  # shift invariance
    g, b = rng.standard_normal(48), rng.standard_normal(48)
    _, ex3 = run(prog, x=x, gamma=g, beta=b)
    want = torch.nn.functional.layer_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), torch.from_numpy(b),
                                          eps=eps).numpy()
    np.testing.assert_allclose(ex3["y"], want, rtol=1e-11, atol=1e-13)


# ------------------------------------------------------------------ RoPE

def _rope(x1, x2, cos, sin):
    _, ex = run(W.get_program("c5_rope"), x1=x1, x2=x2, cos=cos, sin=sin)
    return ex["y1"], ex["y2"]


def test_rope_invariants():
    rng = np.random.default_rng(11)
    T, Hh, D = 5, 3, 8
    x1, x2 = rng.standard_normal((T, Hh, D)), rng.standard_normal((T, Hh, D))
    th = rng.uniform(-3, 3, (T, 1, D))
    y1, y2 = _rope(x1, x2, np.ones((T, 1, D)), np.zeros((T, 1, D)))
    assert np.array_equal(y1, x1) and np.array_equal(y2, x2)            # identity rotation, bit exact
    y1, y2 = _rope(x1, x2, np.cos(th), np.sin(th))
    np.testing.assert_allclose(y1 ** 2 + y2 ** 2, x1 ** 2 + x2 ** 2, rtol=1e-13)   # norm per pair
    q1, q2 = _rope(x1, x2, np.zeros((T, 1, D)), np.ones((T, 1, D)))     # theta = pi/2: (x1,x2)->(-x2,x1)
    assert np.array_equal(q1, -x2) and np.array_equal(q2, x1)
    th2 = rng.uniform(-3, 3, (T, 1, D))
    z1, z2 = _rope(y1, y2, np.cos(th2), np.sin(th2))                    # composition adds angles
    w1, w2 = _rope(x1, x2, np.cos(th + th2), np.sin(th + th2))
    np.testing.assert_allclose(z1, w1, atol=1e-13)
    np.testing.assert_allclose(z2, w2, atol=1e-13)
    # complex-number statement of the same rotation
    zc = (x1 + 1j * x2) * np.exp(1j * th)
    np.testing.assert_allclose(y1, zc.real, atol=1e-14)
    np.testing.assert_allclose(y2, zc.imag, atol=1e-14)


# ------------------------------------------------------------------ config-4 chain

def _c4(T=3, H=32, seed=0, **over):
    rng = np.random.default_rng(seed)
    bf = lambda a: interp.round_to_bf16(a)
    d = dict(x=bf(rng.standard_normal((T, H))), r=bf(rng.standard_normal((T, H))),
             gamma=bf(1 + 0.1 * rng.standard_normal(H)), beta=bf(0.1 * rng.standard_normal(H)),
             bias=bf(0.1 * rng.standard_normal(H)),
             mask=bf(np.where(rng.uniform(size=(T, H)) < 0.9, 1 / 0.9, 0.0)))
    d.update(over)
    return d


def test_c4_chain_special_cases():
    prog = W.get_program("c4_chain")
    d = _c4(mask=np.zeros((3, 32)))
    r, _ = run(prog, **d)
    assert np.array_equal(r["y"], interp.round_to_bf16(d["x"] + d["r"]))     # mask = 0 -> bf16(x + r)
    d = _c4(gamma=np.zeros(32), beta=np.zeros(32), bias=np.zeros(32))
    r, _ = run(prog, **d)
    assert np.array_equal(r["y"], interp.round_to_bf16(d["x"] + d["r"]))     # gelu(0) = 0 -> bf16(h)
    # spelled-out chain == chain with the compound LayerNorm op == torch float64 eager
    d = _c4(T=4, H=64, seed=3)
    _, e1 = run(prog, **d)
    _, e2 = run(W.get_program("c4_chain_ln"), **d)
    np.testing.assert_allclose(e1["y"], e2["y"], rtol=1e-13, atol=1e-15)
    t = {k: torch.from_numpy(v) for k, v in d.items()}
    h = t["x"] + t["r"]
    F = torch.nn.functional
    want = F.gelu(F.layer_norm(h, (64,), t["gamma"], t["beta"], 1e-5) + t["bias"], approximate="tanh") * t["mask"] + h
    np.testing.assert_allclose(e1["y"], want.numpy(), rtol=1e-11, atol=1e-13)
    assert set(np.unique(d["mask"])) <= {0.0, 1.109375}                     # the stored bf16 mask value


def test_outputs_are_rounded_once_to_storage():
    d = _c4()
    r, e = run(W.get_program("c4_chain"), **d)
    assert np.array_equal(r["y"], interp.round_to_bf16(e["y"]))
    x = np.array([[1.0 + 2.0 ** -30, 3.0]])
    r, e = run(W.get_program("identity_affine"), x=x)
    assert r["y"][0, 0] == 1.0 and e["y"][0, 0] != 1.0


def test_add_sqrt_example_and_if_else_add():
    # the paper's vector-vector fusion example c = a + b, d = sqrt(c) (Section 5.1)
    a, b = np.array([[1.0, 7.0]]), np.array([[3.0, 9.0]])
    _, e = run(W.get_program("add_sqrt"), a=a, b=b)
    assert e["d"].tolist() == [[2.0, 4.0]]
    # (a > b ? 2x : 4x) + y  (Section 6, Datasets)
    a, b = np.array([1.0, 2.0, 3.0]), np.array([2.0, 2.0, 2.0])
    x, y = np.array([10.0, 20.0, 30.0]), np.array([1.0, 1.0, 1.0])
    _, e = run(W.get_program("if_else_add"), a=a, b=b, x=x, y=y)
    assert e["o"].tolist() == [41.0, 81.0, 61.0]
    _, et = run(W.get_program("if_else_add_true"), x=x, y=y)
    _, ef = run(W.get_program("if_else_add_false"), x=x, y=y)
    assert et["o"].tolist() == [21.0, 41.0, 61.0] and ef["o"].tolist() == [41.0, 81.0, 121.0]


# ------------------------------------------------------------------ reductions along the penultimate axis (Table 1)

def test_penultimate_axis_reductions_closed_form_and_bruteforce():
    # closed form: x[m, r, n] = r * (n + 1) + m  =>  sum_r = (n + 1) * size * (size - 1) / 2 + m * size,
    # max_r = (size - 1) * (n + 1) + m, min_r = m; a transposed or wrong-axis reduction fails the shape
    # or the values (M, size and N all differ)
    M, size, N = 3, 7, 5
    m, r, n = np.meshgrid(np.arange(M), np.arange(size), np.arange(N), indexing="ij")
    x = (r * (n + 1) + m).astype(np.float64)
    nn = np.arange(N, dtype=np.float64)
    mm = np.arange(M, dtype=np.float64)[:, None, None]
    for op, want in (("csum", (nn + 1) * size * (size - 1) / 2 + mm * size),
                     ("cmax", (size - 1) * (nn + 1) + mm + 0 * nn),
                     ("cmin", mm + 0 * nn)):
        _, ex = run(single_op_program(op, 1), a0=x)
        assert ex["y"].shape == (M, 1, N)
        assert np.array_equal(ex["y"], np.broadcast_to(want, (M, 1, N))), op
    # brute force with plain loops on random values
    rng = np.random.default_rng(41)
    x = rng.standard_normal((2, 6, 4)).astype(np.float32).astype(np.float64)
    _, s = run(single_op_program("csum", 1), a0=x)
    _, hi = run(single_op_program("cmax", 1), a0=x)
    _, lo = run(single_op_program("cmin", 1), a0=x)
    for i in range(2):
        for k in range(4):
            col = [x[i, j, k] for j in range(6)]
            assert s["y"][i, 0, k] == pytest.approx(math.fsum(col), rel=1e-15, abs=1e-15)
            assert hi["y"][i, 0, k] == max(col)
            assert lo["y"][i, 0, k] == min(col)
    # N = 1 is the row reduction: the same numbers as `sum` over the last axis of the transposed input
    x1 = rng.standard_normal((3, 9, 1))
    _, a = run(single_op_program("csum", 1), a0=x1)
    _, b = run(single_op_program("sum", 1), a0=np.swapaxes(x1, -1, -2).copy())
    assert np.allclose(a["y"], b["y"], rtol=1e-15)
    # rank 2: [size, N] -> [1, N], checked against torch's fp64 reduction
    x2 = rng.standard_normal((11, 3))
    _, c = run(single_op_program("csum", 1), a0=x2)
    assert np.allclose(c["y"], torch.from_numpy(x2).sum(dim=0, keepdim=True).numpy(), rtol=1e-14)
