"""The library's host-side inspection (unit_inspect) against the oracle, field by field.

Host logic only: runs without a GPU.  Discrete results, so the bar is equality.
"""
import numpy as np
import pytest

from oracle import inspector as oi
from paper_2101_08458_amd import tensor_programs as tp
from paper_2101_08458_amd import unit


def _same(itext, otext):
    got = unit.unit_inspect(itext, otext)
    ref = oi.inspect(itext, otext)
    ref = dict(ref, operands=[(a, b, list(c)) for a, b, c in ref["operands"]])
    assert got == ref, (itext, otext, got, ref)
    return got


def test_paper_examples():
    assert _same(tp.VNNI, tp.paper_conv())["mapping"] == {"i": "k", "j": "rc"}
    _same(tp.VNNI, tp.paper_conv(act="i8"))
    _same(tp.ARM_DOT, tp.paper_conv(act="i8"))
    _same(tp.TENSOR_CORE, tp.matmul(64, 64, 64))
    _same(tp.TENSOR_CORE, tp.matmul(64, 64, 64, b_transposed=True))
    _same(tp.TENSOR_CORE, tp.matmul(64, 64, 64, accum="f16"))
    _same(tp.TENSOR_CORE, tp.paper_conv(act="f16", wgt="f16", accum="f32"))


@pytest.mark.parametrize("dtype", [unit.UNIT_I8, unit.UNIT_F16])
@pytest.mark.parametrize("edge", [32, 16])
def test_mapping_the_kernels_hard_wire(dtype, edge):
    # The main kernel puts output channels (matmul m) on MFMA rows, pixels (matmul n) on MFMA
    # columns and input channels on the MFMA reduction; the inspection must derive exactly that
    # from the descriptions of the instruction and of the operation.
    mfma = unit.unit_describe_mfma(dtype, edge)
    conv = unit.unit_describe_conv2d(unit.conv_desc(2, 96, 28, 28, 160, 3, 3, (2, 2), (1, 1)), dtype)
    res = _same(mfma, conv)
    assert res["applicable"] and res["mapping"] == {"i": "k", "j": "q", "kk": "c"}
    assert res["operands"] == [("d", "y", []), ("a", "wp", []), ("b", "xp", [])]
    mm = unit.unit_describe_matmul(512, 384, 1024, dtype)
    res = _same(mfma, mm)
    assert res["mapping"] == {"i": "m", "j": "n", "kk": "k"} and res["num_feasible"] == 1
    # an int8 instruction does not apply to an fp16 operation and vice versa
    other = unit.UNIT_F16 if dtype == unit.UNIT_I8 else unit.UNIT_I8
    assert _same(mfma, unit.unit_describe_matmul(64, 64, 64, other))["failed_step"] == 1


def test_mfma_reduction_depths():
    # 16 operand bytes per lane: k = 32 / 64 bytes for the 32- / 16-edge tile
    assert "loop kk 32 red" in unit.unit_describe_mfma(unit.UNIT_I8, 32)
    assert "loop kk 64 red" in unit.unit_describe_mfma(unit.UNIT_I8, 16)
    assert "loop kk 16 red" in unit.unit_describe_mfma(unit.UNIT_F16, 32)
    assert "loop kk 32 red" in unit.unit_describe_mfma(unit.UNIT_F16, 16)


@pytest.mark.parametrize("seed", range(8))
def test_random_programs(seed):
    g = np.random.default_rng(977 + seed)
    kinds = {0: 0, 1: 0, 2: 0}
    for _ in range(150):
        itext, otext = tp.random_program_pair(g)
        kinds[_same(itext, otext)["failed_step"]] += 1
    assert all(v > 0 for v in kinds.values()), kinds


def test_errors():
    good = "loop i 4 dp\nout d:i32[i]\nbody a:i32[i]"
    for bad in ("", "loop i 4 dp\nbody a:i32[i]", "loop i 4 dp\nout d:i32[z]\nbody a:i32[i]",
                "loop i 0 dp\nout d:i32[i]\nbody a:i32[i]", "loop i 4 xx\nout d:i32[i]\nbody a:i32[i]",
                "loop i 4 dp\nout d:i32[i]\nbody (mul a:i32[i])", "loop i 4 dp\nout d:i32[i]\nbody a:i32[i] junk",
                "loop i 4 dp; loop i 4 dp\nout d:i32[i]\nbody a:i32[i]"):
        with pytest.raises(unit.UnitError):
            unit.unit_inspect(bad, good)
        with pytest.raises(unit.UnitError):
            unit.unit_inspect(good, bad)
        if bad:
            with pytest.raises(oi.ParseError):
                oi.parse(bad)
    many = "; ".join(f"loop i{t} 2 dp" for t in range(9)) + "\nout d:i32[i0]\nbody a:i32[i0]"
    with pytest.raises(unit.UnitError):
        unit.unit_inspect(many, many)
    with pytest.raises(unit.UnitError):
        unit.unit_describe_mfma(unit.UNIT_I8, 8)
    with pytest.raises(unit.UnitError):
        unit.unit_describe_matmul(0, 4, 4, unit.UNIT_I8)
