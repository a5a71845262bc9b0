"""Parity of the HIP virtual machine against the CPU oracle on NaN, infinities, signed zeros and negative
bases: Table 1's Min / Max (element-wise and as reductions along the last and the penultimate axis) propagate a
NaN operand, Pow follows the C library's pow on negative bases, zeros and infinities."""
import sys

import numpy as np
import pytest
import torch

from tests import harness as H
from workloads import gen
from workloads.programs import _p, single_op_program

pytestmark = pytest.mark.gpu
DEV = "cuda"
NAN, INF = float("nan"), float("inf")


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


def _special(shape, seed):
    """N(0,1) values with NaN, +-inf and -0 planted at fixed places of every row."""
    x = gen.randn(shape, seed, DEV)
    flat = x.view(-1, shape[-1])
    n = shape[-1]
    flat[:, 3 % n] = -0.0
    flat[0::4, 7 % n] = NAN
    flat[1::4, 11 % n] = INF
    flat[2::4, 13 % n] = -INF
    flat[3::4, (n - 1)] = NAN        # the last element of a row (the ragged chunk when n is not a multiple of 4)
    return x


@pytest.mark.parametrize("op", ["min", "max"])
@pytest.mark.parametrize("cols", [256, 1001])
def test_elementwise_min_max_propagate_nan(op, cols):
    say("elementwise", op, "with NaN / inf / -0, cols", cols)
    a = _special((12, cols), 9100)
    b = gen.randn((12, cols), 9101, DEV)
    b[:, 5] = NAN
    b[:, 7] = 1.0          # NaN on the left only
    for x, y in ((a, b), (b, a)):
        outs, _, _ = H.check_program(single_op_program(op, 2), {"a0": x, "a1": y})
        want = torch.isnan(x) | torch.isnan(y)
        assert torch.equal(torch.isnan(outs["y"]), want)


@pytest.mark.parametrize("op", ["rmax", "rmin"])
@pytest.mark.parametrize("cols", [64, 100, 4096, 5003, 8192])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_row_max_min_propagate_nan(op, cols, dtype):
    say("row", op, "with NaN / inf / -0, cols", cols, dtype)
    x = _special((16, cols), 9200 + cols)
    x[5] = gen.randn((cols,), 9300, DEV)        # a row without special values
    x[6, :] = -INF
    x[6, cols // 2] = 2.0
    if dtype == "bf16":
        x = x.to(torch.bfloat16)
    outs, _, _ = H.check_program(single_op_program(op, 1, dtype), {"a0": x})
    got_nan = torch.isnan(outs["y"]).flatten()
    assert torch.equal(got_nan, torch.isnan(x.float()).any(dim=-1))


@pytest.mark.parametrize("op", ["cmax", "cmin"])
@pytest.mark.parametrize("shape", [(3, 37, 300), (2, 600, 72), (1, 4100, 520)], ids=lambda s: "x".join(map(str, s)))
def test_column_max_min_propagate_nan(op, shape):
    # (few units and a long reduced axis take the streaming record, the others go row by row)
    say("column", op, "with NaN / inf / -0", shape)
    x = gen.randn(shape, 9400 + shape[1], DEV)
    x[0, 5, 7] = NAN
    x[-1, shape[1] - 1, shape[2] - 1] = NAN
    x[0, 2, 9] = INF
    x[0, 3, 9] = -INF
    x[0, :, 11] = -0.0
    desc = _p("col_" + op, [("x", "f32")], [("y", op, ["x"], {})], [("y", "f32")])
    outs, _, _ = H.check_program(desc, {"x": x})
    assert torch.equal(torch.isnan(outs["y"]), torch.isnan(x).any(dim=-2, keepdim=True))


def test_softmax_row_with_nan_is_all_nan():
    say("softmax fp32 with a NaN in some rows")
    z = gen.randn((8, 777), 9500, DEV)
    z[2, 100] = NAN
    z[5, 776] = NAN
    outs, _, _ = H.check_program(single_op_program("softmax", 1), {"a0": z})
    assert torch.isnan(outs["y"][2]).all() and torch.isnan(outs["y"][5]).all() and not torch.isnan(outs["y"][0]).any()


def test_pow_negative_bases_and_special_cases():
    say("pow: negative bases with integer and fractional exponents, zeros, infinities, NaN")
    bases = [-8.0, -2.5, -1.0, -0.5, -0.0, 0.0, 0.5, 1.0, 2.0, 9.0, INF, -INF, NAN]
    exps = [-3.0, -2.0, -1.0, -0.5, -0.0, 0.0, 0.5, 1.0, 2.0, 3.0, 4.0, 2.5, 17.0, INF, -INF, NAN]
    a = torch.tensor(bases, device=DEV).view(-1, 1).expand(len(bases), len(exps)).contiguous()
    b = torch.tensor(exps, device=DEV).view(1, -1).expand(len(bases), len(exps)).contiguous()
    outs, _, _ = H.check_program(single_op_program("pow", 2), {"a0": a, "a1": b})
    y = outs["y"].cpu()
    ref = np.power(a.cpu().numpy().astype(np.float64), b.cpu().numpy().astype(np.float64))
    assert np.array_equal(np.isnan(y.numpy()), np.isnan(ref))
    # x ** 2 and x ** 3 on a tensor of both signs, exponent as a broadcast operand
    x = gen.randn((9, 515), 9600, DEV, std=3.0)
    for e in (2.0, 3.0, -1.0, 5.0):
        H.check_program(single_op_program("pow", 2), {"a0": x, "a1": torch.full((1,), e, device=DEV)})
