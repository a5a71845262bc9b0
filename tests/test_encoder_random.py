"""Random programs through the host side only: every program either encodes into bytecode that
validates, disassembles and is reproduced byte for byte by a second encode, or is refused with an
error code (never a crash)."""
import pytest

from paper_2603_24239_amd import binding as B

from . import random_programs as R

ACCEPTED_REFUSALS = {-5, -4}        # unsupported by the VM, rank


def _shapes(desc, specs):
    out = []
    for n, _ in desc.inputs:
        shape, _dt, layout = specs[n]
        out.append(B.make_shape(shape, R.layout_of(shape, layout)))
    return out


def test_random_programs_encode_or_refuse_cleanly():
    ctx = B.Context(-1)
    lim = B.Context(-1)
    lim.set_limits(16, 4)
    ok = refused = 0
    for seed in range(400):
        desc, specs, dom, _ = R.make(seed)
        prog = B.Program(desc)
        for c in (ctx, lim):
            try:
                code = B.dvm_encode(c, prog, _shapes(desc, specs), None)
            except B.DvmError as e:
                assert e.status in ACCEPTED_REFUSALS, (seed, str(e))
                refused += 1
                continue
            code.validate()
            assert code.disasm()
            again = B.dvm_encode(c, prog, _shapes(desc, specs), None)
            assert again.raw == code.raw, seed
            inf = code.info()
            assert inf.block <= 1024 and inf.grid >= (1 if inf.n_tiles else 0)
            if c is lim:
                assert inf.variant_k <= 16 and inf.variant_nr <= 4
            ok += 1
    assert ok >= 0.8 * (ok + refused), (ok, refused)
